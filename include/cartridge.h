/*
 * cartridge.h -- C ABI of the MI355X (gfx950) hot path of Cartridge / Self-Study training
 * (arxiv 2506.06266).  C11; no HIP or PyTorch types appear here.
 *
 * Conventions shared by every entry point
 *   - Every data pointer is a DEVICE pointer, 16-byte aligned, to a dense row-major tensor in the
 *     layout stated at the entry point.  Descriptors are HOST structs passed by pointer.
 *   - The caller owns every buffer, including the workspace; the library never allocates, frees
 *     or synchronises.  All work is enqueued on `stream` (a hipStream_t passed as void*, NULL is
 *     the default stream); outputs are valid once the caller has synchronised that stream.
 *   - Arguments are validated on the host before anything is launched.  On any error the
 *     matching status is returned and nothing is enqueued; nothing is thrown across the ABI.
 *   - Data-shaped outputs (O, dQ, dK_own, dV_own, d_logits) have the input dtype, rounded from
 *     fp32 to nearest-even; reductions that feed an optimiser or a merge (dZ, loss, LSE, row_kl)
 *     are fp32.  All accumulation is fp32.
 *   - Query head h reads KV head h / (Hq / Hkv).  Q and K arrive with positional encoding already
 *     applied; Z_k is used as stored.
 */
#ifndef CARTRIDGE_H
#define CARTRIDGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CART_OK = 0,
    CART_ERR_NULL = 1,        /* a required pointer is NULL */
    CART_ERR_SHAPE = 2,       /* a size is negative / zero where it may not be, or sizes disagree */
    CART_ERR_UNSUPPORTED = 3, /* dtype / head_dim / mode not implemented */
    CART_ERR_WORKSPACE = 4,   /* workspace NULL or smaller than the *_workspace() query */
    CART_ERR_LAUNCH = 5,      /* the HIP runtime refused a launch */
    CART_ERR_ALIGN = 6        /* a pointer is not 16-byte aligned */
} cart_status;

typedef enum { CART_F32 = 0, CART_BF16 = 1 } cart_dtype;

/* Which kernels serve an attention call.  AUTO picks the MFMA kernels when the shape allows
 * (bf16, head_dim 128) and the fp32 vector kernels otherwise. */
typedef enum { CART_IMPL_AUTO = 0, CART_IMPL_VECTOR = 1, CART_IMPL_MFMA = 2 } cart_impl;

/* One layer's cartridge attention problem (Sec. 3.2: trainable pairs first, then own pairs). */
typedef struct {
    int32_t B;              /* sequences in the batch, >= 1 */
    int32_t S;              /* tokens per sequence, >= 1 */
    int32_t Hq;             /* query heads */
    int32_t Hkv;            /* key/value heads, divides Hq */
    int32_t D;              /* head_dim: 1..256 (vector kernels), 128 (MFMA kernels) */
    int32_t P;              /* prefix (cartridge) slots p, >= 0; 0 is plain causal attention */
    cart_dtype dtype;       /* dtype of Q, K, V, Z, O, dO and of dQ, dK_own, dV_own */
    float softmax_scale;    /* multiplies q.k; 0 selects 1/sqrt(D) */
    int32_t n_frozen;       /* backward: dZ rows [0, n_frozen) are written as 0 (App. A.1, frozen
                               attention-sink slot); 0 <= n_frozen <= P */
    int32_t dz_accumulate;  /* backward: 0 overwrites d_z_k / d_z_v, 1 adds into them */
    cart_impl impl;
} cart_attn_desc;

/* What Eq. 3 becomes when only the teacher's top entries were recorded (App. A.2):
 *   CART_KL_TOPK  the terms of the recorded tokens only (the unrecorded tail is dropped);
 *   CART_KL_REST  the recorded tokens plus one extra outcome "every other token" on both sides,
 *                 i.e. the KL divergence of the two (K+1)-outcome distributions. */
typedef enum { CART_KL_TOPK = 0, CART_KL_REST = 1 } cart_kl_mode;

/* Context-distillation loss over N positions (Eq. 3, Sec. 4.2). */
typedef struct {
    int32_t N;              /* positions (rows), >= 1 */
    int32_t V;              /* vocabulary size, >= 1 */
    int32_t K;              /* recorded teacher entries per position, 1..V and <= 1024 */
    cart_dtype logits_dtype;
    float scale;            /* loss = scale * sum_n KL_n (1/N gives the mean) */
    cart_kl_mode mode;      /* which divergence over the recorded entries; 0 = CART_KL_TOPK */
} cart_kl_desc;

/* Serve-time decode step over a shared cartridge (Sec. 3.3). */
typedef struct {
    int32_t B;                  /* requests, >= 1 */
    int32_t Hq, Hkv, D, P;      /* as in cart_attn_desc */
    int32_t total_own_tokens;   /* T = cu_lens[B]; sizes the even split of the packed own rows (rows
                                   past a smaller value would go unattended) */
    int32_t max_own_len;        /* upper bound on any request's own length (sizes the split) */
    cart_dtype dtype;
    float softmax_scale;        /* 0 selects 1/sqrt(D) */
    cart_impl impl;
} cart_decode_desc;

/* Teacher records over N positions (App. A.2): the K most probable tokens of each. */
typedef struct {
    int32_t N;              /* positions (rows), >= 1 */
    int32_t V;              /* vocabulary size, >= 1 */
    int32_t K;              /* records per position, 1..min(V, 1024) */
    cart_dtype logits_dtype;
} cart_topk_desc;

/* One trained cartridge (or a piece of one): key and value vectors [Hkv,p,D], device memory. */
typedef struct {
    const void *z_k;
    const void *z_v;
    int32_t p;              /* slots, >= 0 (an empty segment adds nothing) */
} cart_segment;
#define CART_MAX_SEGMENTS 8

/* Decode step over composed cartridges (Sec. 5.4) and / or one cartridge per request (the
 * serving protocol of App. A.3, "Throughput measurement details"). */
typedef struct {
    int32_t B;                  /* requests, >= 1 */
    int32_t Hq, Hkv, D;         /* as in cart_attn_desc */
    int32_t n_shared;           /* 0..CART_MAX_SEGMENTS segments every request attends over */
    int32_t n_pool;             /* cartridges in the per-request pool, 0 = no pool */
    int32_t pool_p;             /* slots of each pooled cartridge (all the same size), >= 1 with a pool */
    int32_t total_own_tokens;   /* T = cu_lens[B]; sizes the even split of the packed own rows (rows
                                   past a smaller value would go unattended) */
    int32_t max_own_len;        /* upper bound on any request's own length */
    cart_dtype dtype;           /* CART_BF16 with D = 128 and Hq/Hkv <= 32 (else CART_ERR_UNSUPPORTED) */
    float softmax_scale;        /* 0 selects 1/sqrt(D) */
} cart_decode_composed_desc;

/* A packed batch of sequences of different lengths for cart_attn_varlen_fwd / _bwd (the
 * training batches of Fig. "Scaling Self-Study compute" hold 64 conversations of at most 1024
 * tokens; the paper does not say how they are laid out -- concatenating them instead of padding
 * is this library's choice). */
typedef struct {
    int32_t T;              /* packed rows = sum of the sequence lengths, >= 1 */
    int32_t B;              /* sequences, >= 1 */
    int32_t max_seqlen;     /* an upper bound of every sequence length, 1 <= max_seqlen <= T */
    int32_t Hq, Hkv, D, P;  /* as in cart_attn_desc; D = 128 */
    cart_dtype dtype;       /* CART_BF16 */
    float softmax_scale;    /* 0 selects 1/sqrt(D) */
    int32_t n_frozen;       /* as in cart_attn_desc */
    int32_t dz_accumulate;  /* as in cart_attn_desc */
} cart_attn_varlen_desc;

/* Bytes of workspace each entry point needs for the given descriptor (0 on an invalid one).  The
 * decode figures depend on the number of CUs of the current device as well (the own-KV part is cut
 * into as many ranges as the chip keeps wavefronts resident): ask with the device current that the
 * call will run on. */
size_t cart_attn_fwd_workspace(const cart_attn_desc *desc);
size_t cart_attn_bwd_workspace(const cart_attn_desc *desc);
size_t cart_attn_varlen_fwd_workspace(const cart_attn_varlen_desc *desc);
size_t cart_attn_varlen_bwd_workspace(const cart_attn_varlen_desc *desc);
size_t cart_kl_workspace(const cart_kl_desc *desc);
size_t cart_decode_workspace(const cart_decode_desc *desc);
size_t cart_decode_composed_workspace(const cart_decode_composed_desc *desc, const cart_segment *shared);

/*
 * cart_attn_fwd -- Eq. 1 (Sec. 2.3) over the cartridge cache of Sec. 3.2.
 * For sequence b, query head h (KV head hk = h / (Hq/Hkv)) and token i, the keys are
 * [ z_k[hk][0..P) ; k_own[b][0..i][hk] ] (every prefix slot visible, own tokens j <= i) and
 *   o[b,i,h]   = sum_j softmax_j(scale * q[b,i,h] . key_j) value_j
 *   lse[b,h,i] = log sum_j exp(scale * q[b,i,h] . key_j).
 *   q      [B,S,Hq,D]   in      k_own, v_own [B,S,Hkv,D] in      z_k, z_v [Hkv,P,D] in
 *   o      [B,S,Hq,D]   out     lse          [B,Hq,S] fp32 out
 * z_k / z_v may be NULL when P == 0.  No output may alias an input.
 */
cart_status cart_attn_fwd(const cart_attn_desc *desc, const void *q, const void *k_own,
                          const void *v_own, const void *z_k, const void *z_v, void *o,
                          float *lse, void *workspace, size_t workspace_bytes, void *stream);

/*
 * cart_attn_bwd -- gradient of cart_attn_fwd (Sec. 3.2: the loss is back-propagated into the
 * key and value vectors of Z with the model frozen).  Given d_o = dLoss/dO and the forward's o
 * and lse:  P_ij = exp(s_ij - lse_i), D_i = d_o_i . o_i, dP_ij = d_o_i . value_j,
 * dS_ij = P_ij (dP_ij - D_i);  dQ_i = scale sum_j dS_ij key_j;  dKey_j = scale sum_i dS_ij q_i;
 * dValue_j = sum_i P_ij d_o_i, where sum_i runs over the rows and the Hq/Hkv query heads that
 * see key j, and for prefix slots additionally over all B sequences.
 *   d_q [B,S,Hq,D] out;  d_k_own, d_v_own [B,S,Hkv,D] out (input dtype)
 *   d_z_k, d_z_v [Hkv,P,D] fp32 out (overwritten, or added into when dz_accumulate = 1; rows
 *   below n_frozen are written as 0 / left untouched when accumulating).
 * d_z_k / d_z_v / z_k / z_v may be NULL when P == 0.  Results are bit-reproducible run to run:
 * the sum over the batch is taken as fp32 partials per chunk of token rows (workspace) added in a
 * fixed order by a reduction kernel.  There is no atomic mode: an fp32 atomic-add epilogue into
 * d_z_* was measured at the Llama-8B shape (B16 S2048 P4096) and was slower in total -- key-
 * stationary kernel 4.55 ms against 4.40-4.44 ms, clearing d_z_* plus the tail 0.017 ms against
 * the reduction kernel's 0.022 ms -- and gives up run-to-run identical results.
 */
cart_status cart_attn_bwd(const cart_attn_desc *desc, const void *q, const void *k_own,
                          const void *v_own, const void *z_k, const void *z_v, const void *o,
                          const float *lse, const void *d_o, void *d_q, void *d_k_own,
                          void *d_v_own, float *d_z_k, float *d_z_v, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * cart_distill_kl_fwd_bwd -- Eq. 3 (Sec. 4.2) restricted to the teacher's recorded top entries
 * (App. A.2 "Training Objective"), fused with its gradient.  Per position n, with
 * t_j = exp(teacher_logp[n,j]), M_n = sum_j t_j and log s = log_softmax(logits[n,:]):
 *   KL_n = sum_j t_j (teacher_logp[n,j] - log s[teacher_idx[n,j]])
 *   loss = scale * sum_n KL_n
 *   d_logits[n,v] = scale * (M_n s[v] - t_v),  t_v = t_j where v = teacher_idx[n,j], else 0.
 * With mode CART_KL_REST, S_n = sum_j s[teacher_idx[n,j]]:
 *   KL_n = (the sum above) + (1 - M_n) (log(1 - M_n) - log(1 - S_n))
 *   d_logits[n,v] = scale * (s[v] - t_v) on recorded tokens, scale * s[v] (M_n - S_n) / (1 - S_n)
 *   elsewhere (1 - M_n and 1 - S_n are floored at 0 / 2^-24: fp32 cannot resolve less).
 * Next-token cross-entropy (the objective Sec. 4.2 compares with) is the case K = 1,
 * teacher_idx = the label (negative = ignore the position), teacher_logp = NULL.
 *   logits [N,V] in;  teacher_idx [N,K] int32 in (distinct within a row, each < V; an entry < 0
 *   is ignored);  teacher_logp [N,K] fp32 in, NULL = all zero (every recorded t_j is 1)
 *   loss   [1] fp32 out (device);  d_logits [N,V] out, dtype of logits, MAY alias logits;
 *   row_kl [N] fp32 out, may be NULL.
 */
cart_status cart_distill_kl_fwd_bwd(const cart_kl_desc *desc, const void *logits,
                                    const int32_t *teacher_idx, const float *teacher_logp,
                                    float *loss, void *d_logits, float *row_kl, void *workspace,
                                    size_t workspace_bytes, void *stream);

/*
 * cart_decode -- Sec. 2.3 decode step with the cache of Sec. 3.3: one query token per request
 * over [ z_k[hk][0..P) ; k_own[cu_lens[b] .. cu_lens[b+1])[hk] ], all visible (the current
 * token's own key/value is the last own row; every request has at least one own row).  One
 * cartridge is shared by all B requests.
 *   q [B,Hq,D] in;  z_k, z_v [Hkv,P,D] in (NULL allowed when P == 0)
 *   k_own, v_own [T,Hkv,D] in, ragged;  cu_lens [B+1] int32 in (device), cu_lens[0] = 0
 *   o [B,Hq,D] out;  lse [B,Hq] fp32 out, may be NULL.
 */
cart_status cart_decode(const cart_decode_desc *desc, const void *q, const void *z_k,
                        const void *z_v, const void *k_own, const void *v_own,
                        const int32_t *cu_lens, void *o, float *lse, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * cart_decode_static -- cart_decode for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels and bit-identical results, but the partial results of the call live
 * in an array inside the library (32 MiB of device memory per GPU the library runs on, held until
 * the process ends) instead of a caller-supplied workspace; the call allocates nothing.
 *   - bf16 with D = 128 only (the matrix-core decode kernels): CART_ERR_UNSUPPORTED otherwise.
 *   - A problem whose cart_decode_workspace() exceeds cart_decode_static_capacity() is refused
 *     with CART_ERR_WORKSPACE before anything is launched (the 128-request, 8192-slot serving
 *     shape needs 21.1 MB).
 *   - Every call on a GPU uses that GPU's one array: calls that overlap in time on the same GPU
 *     (two streams, two threads) race; calls on one stream do not.  Nothing in it has to be
 *     cleared between calls: every partial result is written before it is read.
 */
cart_status cart_decode_static(const cart_decode_desc *desc, const void *q, const void *z_k,
                               const void *z_v, const void *k_own, const void *v_own,
                               const int32_t *cu_lens, void *o, float *lse, void *stream);
size_t cart_decode_static_capacity(void);

/*
 * cart_teacher_topk -- the producer of cart_distill_kl_fwd_bwd's teacher inputs (App. A.2: the
 * teacher's top output probabilities are collected while it generates).  Per position n:
 *   teacher_idx[n,0..K)  the K tokens with the largest logits, by descending logit, the lower
 *                        token index first among equal logits (so the result is unique);
 *   teacher_logp[n,j]  = logits[n, teacher_idx[n,j]] - log sum_v exp(logits[n,v]).
 *   logits [N,V] in (bf16 or fp32);  teacher_idx [N,K] int32 out;  teacher_logp [N,K] fp32 out.
 * No workspace.  Indices are exact (comparisons on the stored values); log-probabilities carry
 * the rounding of an fp32 log-sum-exp.
 */
cart_status cart_teacher_topk(const cart_topk_desc *desc, const void *logits, int32_t *teacher_idx,
                              float *teacher_logp, void *stream);

/*
 * cart_decode_composed -- cart_decode with the prefix given in pieces.  Request b attends over,
 * in cache order: the n_shared segments of `shared` (Sec. 5.4: cartridges trained independently
 * are composed by concatenating them; no segment is copied), then, when cart_id[b] >= 0, its own
 * cartridge pool_k / pool_v[cart_id[b]], then its own rows; all visible.  With one shared
 * segment and no pool this is cart_decode.
 *   q [B,Hq,D] in;  shared: host array of n_shared segments (device pointers inside), read
 *   during the call only;  pool_k, pool_v [n_pool,Hkv,pool_p,D] in, cart_id [B] int32 in
 *   (device; an entry < 0: no private cartridge; every entry < n_pool) -- all three NULL when
 *   n_pool == 0;  k_own, v_own, cu_lens, o, lse as in cart_decode.
 */
cart_status cart_decode_composed(const cart_decode_composed_desc *desc, const void *q,
                                 const cart_segment *shared, const void *pool_k, const void *pool_v,
                                 const int32_t *cart_id, const void *k_own, const void *v_own,
                                 const int32_t *cu_lens, void *o, float *lse, void *workspace,
                                 size_t workspace_bytes, void *stream);

/*
 * cart_attn_varlen_fwd / cart_attn_varlen_bwd -- cart_attn_fwd / cart_attn_bwd (Eq. 1 over the
 * cache of Sec. 3.2, and its gradient) over a packed batch: sequence b owns rows
 * cu_seqlens[b] .. cu_seqlens[b+1]-1 of the T packed rows and attends over [Z ; its own rows,
 * causally] exactly as one sequence of a cart_attn_fwd batch; d_z_k / d_z_v sum over all
 * sequences.  Sequences never see each other.
 *   q, o, d_o, d_q [T,Hq,D];  k_own, v_own, d_k_own, d_v_own [T,Hkv,D];  z_k, z_v [Hkv,P,D];
 *   lse [Hq,T] fp32;  d_z_k, d_z_v [Hkv,P,D] fp32 (n_frozen / dz_accumulate as in cart_attn_bwd);
 *   cu_seqlens [B+1] int32 in (device): cu_seqlens[0] = 0, non-decreasing, cu_seqlens[B] = T,
 *   no length above max_seqlen.  The library cannot see the array's contents: offsets outside
 *   [0, T] are the caller's error and are not detected; a sequence may be empty.
 * bf16 with D = 128 only (CART_ERR_UNSUPPORTED otherwise).  Other rules as in cart_attn_fwd /
 * cart_attn_bwd.
 */
cart_status cart_attn_varlen_fwd(const cart_attn_varlen_desc *desc, const void *q, const void *k_own,
                                 const void *v_own, const void *z_k, const void *z_v,
                                 const int32_t *cu_seqlens, void *o, float *lse, void *workspace,
                                 size_t workspace_bytes, void *stream);
cart_status cart_attn_varlen_bwd(const cart_attn_varlen_desc *desc, const void *q, const void *k_own,
                                 const void *v_own, const void *z_k, const void *z_v,
                                 const int32_t *cu_seqlens, const void *o, const float *lse,
                                 const void *d_o, void *d_q, void *d_k_own, void *d_v_own,
                                 float *d_z_k, float *d_z_v, void *workspace, size_t workspace_bytes,
                                 void *stream);

/*
 * cart_trace_events -- optional per-kernel timing hook for benchmarks (not part of the paper).
 * `events` is a host array of `count` hipEvent_t handles (passed as void*), or NULL to switch
 * the hook off.  While set, every later cart_attn_fwd / cart_attn_bwd (also the packed
 * variants) / cart_distill_kl_fwd_bwd / cart_decode call records events[0] on its stream before
 * its first kernel and events[i] after its i-th kernel (as many as `count` allows).  Kernel
 * order, bf16 / head_dim 128: attention forward = forward, overflow repair; backward = dQ
 * (which also forms the row statistics), dK + dV (one kernel), the two dZ reductions (one event); loss = row kernel, scalar
 * reduction; decode = prefix + own-KV (one launch), merge.  The array must stay valid while the
 * hook is set.  Process-global, not thread-safe; the caller owns the events and reads them after
 * synchronising the stream.
 */
cart_status cart_trace_events(void *const *events, int32_t count);

/*
 * cart_calib_* -- benchmark hooks (not part of the paper): plain kernels that measure what this
 * machine gives a kernel with nothing else to do, so that a benchmark can put a rate of the hot
 * path next to a peak measured in the same run.  The caller times them with events on `stream`.
 *   cart_calib_mfma  a matrix-core-only loop of the bf16 instruction the attention kernels use
 *                    (register operands, pseudo-random values), wgs_per_cu (1..8) workgroups of
 *                    four wavefronts per CU, `iters` x 8 instructions per wavefront.  Returns the
 *                    floating-point operations the launch performs (0 on a bad argument or a
 *                    refused launch).  sink: 4 bytes of device memory, never written in practice.
 *   cart_calib_copy  dst[0..bytes) = src[0..bytes), 16 bytes per lane per step (bytes % 16 == 0).
 *   cart_calib_read  reads src[0..bytes) the same way; sink as above.
 */
double cart_calib_mfma(void *sink, int32_t iters, int32_t wgs_per_cu, void *stream);
cart_status cart_calib_copy(void *dst, const void *src, size_t bytes, void *stream);
cart_status cart_calib_read(const void *src, size_t bytes, void *sink, void *stream);

const char *cart_status_str(cart_status status);
int cart_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CARTRIDGE_H */
