// C-ABI layer of libcartridge: host-side validation and dispatch.  Nothing is launched unless
// every argument passed validation; the library never allocates or synchronises.
#include <math.h>

#include "cart_common.h"

namespace cart {
Trace& trace() {
    static Trace t;
    return t;
}
}  // namespace cart

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t n) { return (n + 255) & ~static_cast<size_t>(255); }

cart_status check_attn(const cart_attn_desc* d) {
    if (!d) return CART_ERR_NULL;
    if (d->B < 1 || d->S < 1 || d->Hq < 1 || d->Hkv < 1 || d->D < 1 || d->P < 0) return CART_ERR_SHAPE;
    if (d->Hq % d->Hkv != 0) return CART_ERR_SHAPE;
    if (d->n_frozen < 0 || d->n_frozen > d->P) return CART_ERR_SHAPE;
    if (d->dtype != CART_F32 && d->dtype != CART_BF16) return CART_ERR_UNSUPPORTED;
    if (d->D > 256) return CART_ERR_UNSUPPORTED;
    if (d->impl != CART_IMPL_AUTO && d->impl != CART_IMPL_VECTOR && d->impl != CART_IMPL_MFMA)
        return CART_ERR_UNSUPPORTED;
    if (d->impl == CART_IMPL_MFMA && !cart::attn_mfma_supported(*d)) return CART_ERR_UNSUPPORTED;
    if (!(d->softmax_scale >= 0.f) || isinf(d->softmax_scale)) return CART_ERR_SHAPE;
    if (static_cast<long>(d->B) * d->S * d->Hq * static_cast<long>(d->D) > (1L << 40)) return CART_ERR_SHAPE;
    return CART_OK;
}
inline bool use_mfma(const cart_attn_desc& d) {
    return d.impl != CART_IMPL_VECTOR && cart::attn_mfma_supported(d);
}
inline bool use_mfma_bwd(const cart_attn_desc& d) {
    return d.impl != CART_IMPL_VECTOR && cart::attn_mfma_bwd_supported(d);
}
inline float attn_scale(float s, int D) { return s > 0.f ? s : 1.0f / sqrtf(static_cast<float>(D)); }

// the packed batch as the batched descriptor the kernels take: S = the longest sequence
cart_status check_varlen(const cart_attn_varlen_desc* d, cart_attn_desc* a) {
    if (!d) return CART_ERR_NULL;
    if (d->T < 1 || d->B < 1 || d->max_seqlen < 1 || d->max_seqlen > d->T) return CART_ERR_SHAPE;
    cart_attn_desc x;
    x.B = d->B; x.S = d->max_seqlen; x.Hq = d->Hq; x.Hkv = d->Hkv; x.D = d->D; x.P = d->P;
    x.dtype = d->dtype; x.softmax_scale = d->softmax_scale; x.n_frozen = d->n_frozen;
    x.dz_accumulate = d->dz_accumulate; x.impl = CART_IMPL_MFMA;
    cart_status s = check_attn(&x);
    if (s != CART_OK) return s;
    if (static_cast<long>(d->T) * d->Hq * static_cast<long>(d->D) > (1L << 40)) return CART_ERR_SHAPE;
    *a = x;
    return CART_OK;
}

cart_status check_kl(const cart_kl_desc* d) {
    if (!d) return CART_ERR_NULL;
    if (d->N < 1 || d->V < 1 || d->K < 1 || d->K > d->V) return CART_ERR_SHAPE;
    if (d->K > 1024) return CART_ERR_UNSUPPORTED;
    if (d->logits_dtype != CART_F32 && d->logits_dtype != CART_BF16) return CART_ERR_UNSUPPORTED;
    if (isnan(d->scale) || isinf(d->scale)) return CART_ERR_SHAPE;
    if (d->mode != CART_KL_TOPK && d->mode != CART_KL_REST) return CART_ERR_UNSUPPORTED;
    return CART_OK;
}

cart_status check_decode(const cart_decode_desc* d) {
    if (!d) return CART_ERR_NULL;
    if (d->B < 1 || d->Hq < 1 || d->Hkv < 1 || d->D < 1 || d->P < 0) return CART_ERR_SHAPE;
    if (d->Hq % d->Hkv != 0) return CART_ERR_SHAPE;
    if (d->total_own_tokens < d->B || d->max_own_len < 1 || d->max_own_len > d->total_own_tokens)
        return CART_ERR_SHAPE;
    if (d->dtype != CART_F32 && d->dtype != CART_BF16) return CART_ERR_UNSUPPORTED;
    if (d->D > 256) return CART_ERR_UNSUPPORTED;
    if (d->impl != CART_IMPL_AUTO && d->impl != CART_IMPL_VECTOR && d->impl != CART_IMPL_MFMA)
        return CART_ERR_UNSUPPORTED;
    if (d->impl == CART_IMPL_MFMA && !cart::decode_mfma_supported(*d)) return CART_ERR_UNSUPPORTED;
    if (!(d->softmax_scale >= 0.f) || isinf(d->softmax_scale)) return CART_ERR_SHAPE;
    return CART_OK;
}
inline bool use_mfma(const cart_decode_desc& d) {
    return d.impl != CART_IMPL_VECTOR && cart::decode_mfma_supported(d);
}

#define REQUIRE(p) do { if (!(p)) return CART_ERR_NULL; } while (0)
#define ALIGNED(p) do { if (!aligned16(p)) return CART_ERR_ALIGN; } while (0)

}  // namespace

extern "C" {

size_t cart_attn_fwd_workspace(const cart_attn_desc* d) {
    if (check_attn(d) != CART_OK) return 0;
    return use_mfma(*d) ? cart::attn_mfma_fwd_workspace(*d) : 0;
}

size_t cart_attn_bwd_workspace(const cart_attn_desc* d) {
    if (check_attn(d) != CART_OK) return 0;
    size_t delta = round256(static_cast<size_t>(d->B) * d->Hq * d->S * sizeof(float));
    return delta + (use_mfma_bwd(*d) ? cart::attn_mfma_bwd_workspace(*d) : 0);
}

size_t cart_attn_varlen_fwd_workspace(const cart_attn_varlen_desc* d) {
    cart_attn_desc a;
    if (check_varlen(d, &a) != CART_OK) return 0;
    return cart::attn_mfma_fwd_workspace(a, d->T);
}

size_t cart_attn_varlen_bwd_workspace(const cart_attn_varlen_desc* d) {
    cart_attn_desc a;
    if (check_varlen(d, &a) != CART_OK) return 0;
    return round256(static_cast<size_t>(d->T) * d->Hq * sizeof(float)) + cart::attn_mfma_bwd_workspace(a, d->T);
}

size_t cart_kl_workspace(const cart_kl_desc* d) {
    if (check_kl(d) != CART_OK) return 0;
    return round256(static_cast<size_t>(d->N) * sizeof(float));
}

cart_status cart_teacher_topk(const cart_topk_desc* d, const void* logits, int32_t* teacher_idx,
                              float* teacher_logp, void* stream) {
    if (!d) return CART_ERR_NULL;
    if (d->N < 1 || d->V < 1 || d->K < 1 || d->K > d->V) return CART_ERR_SHAPE;
    if (d->K > 1024) return CART_ERR_UNSUPPORTED;
    if (d->logits_dtype != CART_F32 && d->logits_dtype != CART_BF16) return CART_ERR_UNSUPPORTED;
    REQUIRE(logits); REQUIRE(teacher_idx); REQUIRE(teacher_logp);
    ALIGNED(logits);
    int e = cart::launch_topk(*d, logits, teacher_idx, teacher_logp, static_cast<hipStream_t>(stream));
    return e == 0 ? CART_OK : CART_ERR_LAUNCH;
}

static cart_status check_decode_composed(const cart_decode_composed_desc* d, const cart_segment* shared) {
    if (!d) return CART_ERR_NULL;
    if (d->B < 1 || d->Hq < 1 || d->Hkv < 1 || d->D < 1) return CART_ERR_SHAPE;
    if (d->Hq % d->Hkv) return CART_ERR_SHAPE;
    if (d->n_shared < 0 || d->n_shared > CART_MAX_SEGMENTS) return CART_ERR_SHAPE;
    if (d->n_pool < 0 || (d->n_pool > 0 && d->pool_p < 1)) return CART_ERR_SHAPE;
    if (d->total_own_tokens < d->B || d->max_own_len < 1 || d->max_own_len > d->total_own_tokens) return CART_ERR_SHAPE;
    if (isnan(d->softmax_scale) || isinf(d->softmax_scale) || d->softmax_scale < 0.f) return CART_ERR_SHAPE;
    if (d->n_shared > 0 && !shared) return CART_ERR_NULL;
    for (int s = 0; s < d->n_shared; ++s) {
        if (shared[s].p < 0) return CART_ERR_SHAPE;
        if (shared[s].p > 0 && (!shared[s].z_k || !shared[s].z_v)) return CART_ERR_NULL;
        if ((reinterpret_cast<uintptr_t>(shared[s].z_k) | reinterpret_cast<uintptr_t>(shared[s].z_v)) & 15) return CART_ERR_ALIGN;
    }
    if (!cart::decode_composed_supported(*d)) return CART_ERR_UNSUPPORTED;
    return CART_OK;
}

size_t cart_decode_composed_workspace(const cart_decode_composed_desc* d, const cart_segment* shared) {
    if (check_decode_composed(d, shared) != CART_OK) return 0;
    return cart::decode_composed_workspace(*d, shared);
}

cart_status cart_decode_composed(const cart_decode_composed_desc* d, const void* q, const cart_segment* shared,
                                 const void* pool_k, const void* pool_v, const int32_t* cart_id,
                                 const void* k_own, const void* v_own, const int32_t* cu_lens, void* o,
                                 float* lse, void* workspace, size_t workspace_bytes, void* stream) {
    cart_status s = check_decode_composed(d, shared);
    if (s != CART_OK) return s;
    REQUIRE(q); REQUIRE(k_own); REQUIRE(v_own); REQUIRE(cu_lens); REQUIRE(o);
    if (d->n_pool > 0) { REQUIRE(pool_k); REQUIRE(pool_v); REQUIRE(cart_id); }
    ALIGNED(q); ALIGNED(k_own); ALIGNED(v_own); ALIGNED(o); ALIGNED(pool_k); ALIGNED(pool_v); ALIGNED(workspace);
    const size_t need = cart::decode_composed_workspace(*d, shared);
    if (!workspace || workspace_bytes < need) return CART_ERR_WORKSPACE;
    const float scale = attn_scale(d->softmax_scale, d->D);
    int e = cart::launch_decode_composed(*d, scale, q, shared, pool_k, pool_v, cart_id, k_own, v_own, cu_lens, o,
                                         lse, workspace, static_cast<hipStream_t>(stream));
    return e == 0 ? CART_OK : CART_ERR_LAUNCH;
}

size_t cart_decode_workspace(const cart_decode_desc* d) {
    if (check_decode(d) != CART_OK) return 0;
    return use_mfma(*d) ? cart::decode_mfma_workspace(*d) : 0;
}

cart_status cart_attn_fwd(const cart_attn_desc* d, const void* q, const void* k_own,
                          const void* v_own, const void* z_k, const void* z_v, void* o, float* lse,
                          void* workspace, size_t workspace_bytes, void* stream) {
    cart_status s = check_attn(d);
    if (s != CART_OK) return s;
    REQUIRE(q); REQUIRE(k_own); REQUIRE(v_own); REQUIRE(o); REQUIRE(lse);
    if (d->P > 0) { REQUIRE(z_k); REQUIRE(z_v); }
    ALIGNED(q); ALIGNED(k_own); ALIGNED(v_own); ALIGNED(z_k); ALIGNED(z_v); ALIGNED(o); ALIGNED(lse);
    ALIGNED(workspace);
    const size_t need = cart_attn_fwd_workspace(d);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CART_ERR_WORKSPACE;
    const float scale = attn_scale(d->softmax_scale, d->D);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int e = use_mfma(*d)
                ? cart::launch_attn_fwd_mfma(*d, scale, q, k_own, v_own, z_k, z_v, o, lse, workspace, st)
                : cart::launch_attn_fwd_vector(*d, scale, q, k_own, v_own, z_k, z_v, o, lse, st);
    return e == 0 ? CART_OK : CART_ERR_LAUNCH;
}

cart_status cart_attn_bwd(const cart_attn_desc* d, const void* q, const void* k_own,
                          const void* v_own, const void* z_k, const void* z_v, const void* o,
                          const float* lse, const void* d_o, void* d_q, void* d_k_own,
                          void* d_v_own, float* d_z_k, float* d_z_v, void* workspace,
                          size_t workspace_bytes, void* stream) {
    cart_status s = check_attn(d);
    if (s != CART_OK) return s;
    REQUIRE(q); REQUIRE(k_own); REQUIRE(v_own); REQUIRE(o); REQUIRE(lse); REQUIRE(d_o);
    REQUIRE(d_q); REQUIRE(d_k_own); REQUIRE(d_v_own);
    if (d->P > 0) { REQUIRE(z_k); REQUIRE(z_v); REQUIRE(d_z_k); REQUIRE(d_z_v); }
    ALIGNED(q); ALIGNED(k_own); ALIGNED(v_own); ALIGNED(z_k); ALIGNED(z_v); ALIGNED(o); ALIGNED(lse);
    ALIGNED(d_o); ALIGNED(d_q); ALIGNED(d_k_own); ALIGNED(d_v_own); ALIGNED(d_z_k); ALIGNED(d_z_v);
    ALIGNED(workspace);
    const size_t need = cart_attn_bwd_workspace(d);
    if (!workspace || workspace_bytes < need) return CART_ERR_WORKSPACE;
    const float scale = attn_scale(d->softmax_scale, d->D);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int e = use_mfma_bwd(*d)
                ? cart::launch_attn_bwd_mfma(*d, scale, q, k_own, v_own, z_k, z_v, o, lse, d_o, d_q,
                                             d_k_own, d_v_own, d_z_k, d_z_v, workspace, st)
                : cart::launch_attn_bwd_vector(*d, scale, q, k_own, v_own, z_k, z_v, o, lse, d_o,
                                               d_q, d_k_own, d_v_own, d_z_k, d_z_v, workspace, st);
    return e == 0 ? CART_OK : CART_ERR_LAUNCH;
}

cart_status cart_attn_varlen_fwd(const cart_attn_varlen_desc* d, const void* q, const void* k_own,
                                 const void* v_own, const void* z_k, const void* z_v,
                                 const int32_t* cu_seqlens, void* o, float* lse, void* workspace,
                                 size_t workspace_bytes, void* stream) {
    cart_attn_desc a;
    cart_status s = check_varlen(d, &a);
    if (s != CART_OK) return s;
    REQUIRE(q); REQUIRE(k_own); REQUIRE(v_own); REQUIRE(cu_seqlens); REQUIRE(o); REQUIRE(lse);
    if (d->P > 0) { REQUIRE(z_k); REQUIRE(z_v); }
    ALIGNED(q); ALIGNED(k_own); ALIGNED(v_own); ALIGNED(z_k); ALIGNED(z_v); ALIGNED(o); ALIGNED(lse);
    ALIGNED(workspace);
    const size_t need = cart_attn_varlen_fwd_workspace(d);
    if (!workspace || workspace_bytes < need) return CART_ERR_WORKSPACE;
    int e = cart::launch_attn_fwd_mfma(a, attn_scale(d->softmax_scale, d->D), q, k_own, v_own, z_k, z_v, o, lse,
                                       workspace, static_cast<hipStream_t>(stream), cu_seqlens, d->T);
    return e == 0 ? CART_OK : CART_ERR_LAUNCH;
}

cart_status cart_attn_varlen_bwd(const cart_attn_varlen_desc* d, const void* q, const void* k_own,
                                 const void* v_own, const void* z_k, const void* z_v,
                                 const int32_t* cu_seqlens, const void* o, const float* lse,
                                 const void* d_o, void* d_q, void* d_k_own, void* d_v_own,
                                 float* d_z_k, float* d_z_v, void* workspace, size_t workspace_bytes,
                                 void* stream) {
    cart_attn_desc a;
    cart_status s = check_varlen(d, &a);
    if (s != CART_OK) return s;
    REQUIRE(q); REQUIRE(k_own); REQUIRE(v_own); REQUIRE(cu_seqlens); REQUIRE(o); REQUIRE(lse); REQUIRE(d_o);
    REQUIRE(d_q); REQUIRE(d_k_own); REQUIRE(d_v_own);
    if (d->P > 0) { REQUIRE(z_k); REQUIRE(z_v); REQUIRE(d_z_k); REQUIRE(d_z_v); }
    ALIGNED(q); ALIGNED(k_own); ALIGNED(v_own); ALIGNED(z_k); ALIGNED(z_v); ALIGNED(o); ALIGNED(lse);
    ALIGNED(d_o); ALIGNED(d_q); ALIGNED(d_k_own); ALIGNED(d_v_own); ALIGNED(d_z_k); ALIGNED(d_z_v);
    ALIGNED(workspace);
    const size_t need = cart_attn_varlen_bwd_workspace(d);
    if (!workspace || workspace_bytes < need) return CART_ERR_WORKSPACE;
    int e = cart::launch_attn_bwd_mfma(a, attn_scale(d->softmax_scale, d->D), q, k_own, v_own, z_k, z_v, o, lse,
                                       d_o, d_q, d_k_own, d_v_own, d_z_k, d_z_v, workspace,
                                       static_cast<hipStream_t>(stream), cu_seqlens, d->T);
    return e == 0 ? CART_OK : CART_ERR_LAUNCH;
}

cart_status cart_distill_kl_fwd_bwd(const cart_kl_desc* d, const void* logits,
                                    const int32_t* teacher_idx, const float* teacher_logp,
                                    float* loss, void* d_logits, float* row_kl, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    cart_status s = check_kl(d);
    if (s != CART_OK) return s;
    REQUIRE(logits); REQUIRE(teacher_idx); REQUIRE(loss); REQUIRE(d_logits);   // teacher_logp NULL = zeros
    ALIGNED(logits); ALIGNED(teacher_idx); ALIGNED(teacher_logp); ALIGNED(d_logits); ALIGNED(workspace);
    if (!row_kl && (!workspace || workspace_bytes < cart_kl_workspace(d))) return CART_ERR_WORKSPACE;
    int e = cart::launch_kl(*d, logits, teacher_idx, teacher_logp, loss, d_logits, row_kl, workspace,
                            static_cast<hipStream_t>(stream));
    return e == 0 ? CART_OK : CART_ERR_LAUNCH;
}

cart_status cart_decode(const cart_decode_desc* d, const void* q, const void* z_k, const void* z_v,
                        const void* k_own, const void* v_own, const int32_t* cu_lens, void* o,
                        float* lse, void* workspace, size_t workspace_bytes, void* stream) {
    cart_status s = check_decode(d);
    if (s != CART_OK) return s;
    REQUIRE(q); REQUIRE(k_own); REQUIRE(v_own); REQUIRE(cu_lens); REQUIRE(o);
    if (d->P > 0) { REQUIRE(z_k); REQUIRE(z_v); }
    ALIGNED(q); ALIGNED(z_k); ALIGNED(z_v); ALIGNED(k_own); ALIGNED(v_own); ALIGNED(o); ALIGNED(workspace);
    const size_t need = cart_decode_workspace(d);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CART_ERR_WORKSPACE;
    const float scale = attn_scale(d->softmax_scale, d->D);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int e = use_mfma(*d)
                ? cart::launch_decode_mfma(*d, scale, q, z_k, z_v, k_own, v_own, cu_lens, o, lse, workspace, st)
                : cart::launch_decode_vector(*d, scale, q, z_k, z_v, k_own, v_own, cu_lens, o, lse, st);
    return e == 0 ? CART_OK : CART_ERR_LAUNCH;
}

size_t cart_decode_static_capacity(void) { return cart::decode_static_capacity(); }

cart_status cart_decode_static(const cart_decode_desc* d, const void* q, const void* z_k, const void* z_v,
                               const void* k_own, const void* v_own, const int32_t* cu_lens, void* o,
                               float* lse, void* stream) {
    cart_status s = check_decode(d);
    if (s != CART_OK) return s;
    if (!cart::decode_mfma_supported(*d) || d->impl == CART_IMPL_VECTOR) return CART_ERR_UNSUPPORTED;
    REQUIRE(q); REQUIRE(k_own); REQUIRE(v_own); REQUIRE(cu_lens); REQUIRE(o);
    if (d->P > 0) { REQUIRE(z_k); REQUIRE(z_v); }
    ALIGNED(q); ALIGNED(z_k); ALIGNED(z_v); ALIGNED(k_own); ALIGNED(v_own); ALIGNED(o);
    if (cart::decode_mfma_workspace(*d) > cart::decode_static_capacity()) return CART_ERR_WORKSPACE;
    void* ws = cart::decode_static_scratch();
    if (!ws) return CART_ERR_LAUNCH;
    const float scale = attn_scale(d->softmax_scale, d->D);
    int e = cart::launch_decode_mfma(*d, scale, q, z_k, z_v, k_own, v_own, cu_lens, o, lse, ws,
                                     static_cast<hipStream_t>(stream));
    return e == 0 ? CART_OK : CART_ERR_LAUNCH;
}

cart_status cart_trace_events(void* const* events, int32_t count) {
    if (events && count < 1) return CART_ERR_SHAPE;
    cart::Trace& t = cart::trace();
    t.events = events;
    t.count = events ? count : 0;
    t.next = 0;
    return CART_OK;
}

const char* cart_status_str(cart_status s) {
    switch (s) {
        case CART_OK: return "ok";
        case CART_ERR_NULL: return "a required pointer is NULL";
        case CART_ERR_SHAPE: return "invalid or inconsistent sizes";
        case CART_ERR_UNSUPPORTED: return "dtype, head_dim or mode not supported";
        case CART_ERR_WORKSPACE: return "workspace missing or too small";
        case CART_ERR_LAUNCH: return "kernel launch failed";
        case CART_ERR_ALIGN: return "a pointer is not 16-byte aligned";
    }
    return "unknown status";
}

int cart_version(void) { return 150; }   // 1.5: + cart_decode_static, calibration hooks; backward in two kernels

}  // extern "C"
