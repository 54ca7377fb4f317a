// Cartridge attention forward on the matrix cores (bf16 in, fp32 accumulate, head_dim 128):
// Eq. 1 over the cache of Sec. 3.2, [prefix Z (all visible) ; own keys (causal)].
//
// One 256-thread workgroup = 256 consecutive queries of one (sequence, query head); each of its
// four wavefronts owns 64 of them, kept in registers as MFMA operand fragments.  Keys/values
// stream through LDS in tiles of 64 (prefix tiles first, then own tiles up to the diagonal),
// three buffers, one barrier per tile, consumed as sub-tiles of 32 keys.  Per sub-tile a
// wavefront computes S^T = K Q^T (keys on the D rows, its queries on the D columns), turns it
// into P = 2^(c S - m) per lane (a lane owns one query) and accumulates O^T += V^T P^T with V
// read through the transposing LDS load.
//
// The softmax reference m of a query is fixed once, from its first sub-tile of keys; there is no
// running max and the O accumulators are never rescaled.  exp2 and the fp32 accumulators cover
// 2^+-126 around that reference, so this is exact unless a later score exceeds the first
// sub-tile's maximum by more than ~80 in natural-log units; then the row sum overflows to
// inf/NaN, the workgroup raises a flag, and attn_fwd_repair_kernel recomputes that block of rows
// with a plain running-max loop.  The hot loop is one straight-line block per sub-tile with two
// independent instruction streams: the matrix cores work on S(u+1) and on O += V P(u-1) while the
// vector ALU turns S(u) into P(u).
#include <type_traits>

#include "attn_mfma.h"

namespace cart {
using namespace mfma;

constexpr int FWD_BM = 256;   // queries per workgroup
constexpr int FWD_BN = 64;    // keys per LDS tile, consumed as two sub-tiles of 32
constexpr int FWD_NBUF = 3;
constexpr int FWD_TILE_B = FWD_BN * ROW_B;

struct FwdSmem {
    char k[FWD_NBUF][FWD_TILE_B];
    char v[FWD_NBUF][FWD_TILE_B];
};

__global__ __launch_bounds__(256, 1) void attn_fwd_mfma_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ zk, const bf16_t* __restrict__ zv, bf16_t* __restrict__ o,
    float* __restrict__ lse, int* __restrict__ flags, int B, int S, int Hq, int Hkv, int P,
    float c /* scale*log2(e) */) {
    __shared__ FwdSmem sm;
    __shared__ int sm_bad;
    const int G = Hq / Hkv;
    const int nQt = (S + FWD_BM - 1) / FWD_BM;
    // workgroup -> (query tile, sequence, head).  KV head is the fastest index so that, with 8
    // KV heads, blockIdx % 8 (the XCD a workgroup lands on) is the KV head and each XCD's L2 keeps
    // one head's prefix; the heaviest query tiles (longest causal part) are issued first.
    int id = blockIdx.x;
    const int hk = id % Hkv; id /= Hkv;
    const int g_ = id % G; id /= G;
    const int b = id % B; id /= B;
    const int qt = nQt - 1 - id;
    const int h = hk * G + g_;
    const int lane = threadIdx.x & 63, lg = lane >> 5, lc = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, in a scalar register
    const int q0 = qt * FWD_BM, wrow0 = q0 + 64 * wv;
    if (threadIdx.x == 0) sm_bad = 0;

    // this wavefront's 64 queries as B-operand fragments: column = query, k = head element
    // They are pinned to accumulation registers (the matrix cores read B operands from there
    // directly), which leaves the ordinary vector registers to the softmax arithmetic.
    u32x4 qraw[2][8];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        int qi = wrow0 + 32 * cb + lc;
        qi = qi < S ? qi : S - 1;
        const bf16_t* qp = q + ((static_cast<size_t>(b) * S + qi) * Hq + h) * HD + 8 * lg;
#pragma unroll
        for (int t = 0; t < 8; ++t) qraw[cb][t] = *reinterpret_cast<const u32x4*>(qp + 16 * t);
    }
#ifndef CART_PIN_Q
#define CART_PIN_Q 1
#endif
    auto pin_q = [&]() __attribute__((always_inline)) {
#if CART_PIN_Q
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int t = 0; t < 8; ++t) asm volatile("" : "+a"(qraw[cb][t]));
#endif
    };
#define qf_(cb, t) __builtin_bit_cast(bf16x8, qraw[cb][t])
    pin_q();

    const int nPt = (P + FWD_BN - 1) / FWD_BN;
    const int own_end = min(S, q0 + FWD_BM);
    const int nT = nPt + (own_end + FWD_BN - 1) / FWD_BN;
    const char* zk_b = reinterpret_cast<const char*>(zk) + static_cast<size_t>(hk) * P * ROW_B;
    const char* zv_b = reinterpret_cast<const char*>(zv) + static_cast<size_t>(hk) * P * ROW_B;
    const size_t own_pitch = static_cast<size_t>(Hkv) * ROW_B;
    const char* k_b = reinterpret_cast<const char*>(k) + (static_cast<size_t>(b) * S * Hkv + hk) * ROW_B;
    const char* v_b = reinterpret_cast<const char*>(v) + (static_cast<size_t>(b) * S * Hkv + hk) * ROW_B;

    // tile t -> LDS buffer; branch-free (prefix or own is a scalar select).  Rows past the end
    // of the prefix / the sequence are clamped onto the last valid row and masked later.
    auto issue = [&](int t, int buf) __attribute__((always_inline)) {
        const bool pre = t < nPt;
        const int j0 = (pre ? t : t - nPt) * FWD_BN;
        const int last = (pre ? P : S) - 1;
        const uint32_t pitch = pre ? static_cast<uint32_t>(ROW_B) : static_cast<uint32_t>(own_pitch);
        const char* kb = pre ? zk_b : k_b;
        const char* vb = pre ? zv_b : v_b;
        tile_load_async<FWD_BN>(sm.k[buf], kb, j0, last, pitch);
        tile_load_async<FWD_BN>(sm.v[buf], vb, j0, last, pitch);
    };
    // does sub-tile (tile t, half hb) hold a key that some query of this wavefront must not see?
    auto needs_mask = [&](int t, int hb) __attribute__((always_inline)) {
        return t < nPt ? (t * FWD_BN + 32 * hb + 32 > P) : ((t - nPt) * FWD_BN + 32 * hb + 31 > wrow0);
    };
    // hidden entries of the scores of sub-tile (t, hb) -> NEG_BIG
    auto mask = [&](f32x16 (&x)[2], int t, int hb) __attribute__((always_inline)) {
        const bool own = t >= nPt;
        const int j0 = (own ? t - nPt : t) * FWD_BN + 32 * hb;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            // key j0 + d_row(r, lg) is hidden when it exceeds the lane's last visible key
            const int thr = (own ? wrow0 + 32 * cb + lc : P - 1) - j0 - 4 * lg;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (8 * (r >> 2) + (r & 3) > thr) x[cb][r] = NEG_BIG;
        }
    };

    f32x16 acc[4][2];   // O^T: [head-element block][query block]
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][cb][r] = 0.f;
    // keeps the O accumulators in accumulation registers across the loop's control flow
    auto pin_acc = [&]() __attribute__((always_inline)) {
#ifndef CART_PIN_ACC
#define CART_PIN_ACC 1
#endif
#if CART_PIN_ACC
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) asm volatile("" : "+a"(acc[db][cb]));
#endif
    };
    float m_ref[2], l_run[2] = {0.f, 0.f};
    f32x16 s[2];              // scores, produced by the matrix cores one iteration ahead
    bf16x8 pf[2][2];          // P^T(u-1) as B-operand fragments [query block][k-step]
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) pf[cb][ks] = bf16x8{};

    // Iteration u.  Matrix cores: S^T(u+1) = K Q^T and O^T += V^T(u-1) P^T(u-1).  Vector ALU:
    // P(u) = 2^(c S(u) - m), row sums, bf16 fragments.  The two streams are independent.
    // LDS -> register fragments run one iteration ahead of their use (loop-carried), so their
    // latency is covered by a whole iteration of work whatever the instruction order inside it
    bf16x8 ka[8], va[2][4];
    auto load_k = [&](const char* kt, int r0) __attribute__((always_inline)) {
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) ka[t8] = lds_frag_n(kt, r0 + lc, 16 * t8 + 8 * lg);
    };
    auto load_v = [&](const char* vt, int r0) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) va[ks][db] = lds_frag_t(vt, r0 + 16 * ks, 32 * db, lane);
    };
    // Iteration u, on entry: s = S(u), ka = K fragments of sub-tile u+1, va = V fragments of
    // sub-tile u-1, pf = P(u-1).  buf / nbuf = LDS buffers of the tiles of sub-tiles u / u+2.
    auto stage = [&](int u, int buf, int nbuf) __attribute__((always_inline)) {
        const int hb = u & 1;
        // the scores of sub-tile u move to ordinary registers (their accumulators are reused by
        // the next sub-tile); the rare masked sub-tile is patched here, outside the main block
        f32x16 x[2] = {s[0], s[1]};
        if (needs_mask(u >> 1, hb)) mask(x, u >> 1, hb);
        pin_q();
        pin_acc();
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[cb][r] = 0.f;
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) {
            s[0] = mma(ka[t8], qf_(0, t8), s[0]);
            s[1] = mma(ka[t8], qf_(1, t8), s[1]);
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                acc[db][0] = mma(va[ks][db], pf[0][ks], acc[db][0]);
                acc[db][1] = mma(va[ks][db], pf[1][ks], acc[db][1]);
            }
        // fragments for the next iteration: K of sub-tile u+2, V of sub-tile u
        load_k(sm.k[0] + nbuf * FWD_TILE_B, 32 * hb);
        load_v(sm.v[0] + buf * FWD_TILE_B, 32 * hb);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            float rs = 0.f;
            f32x16 p;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                p[r] = fast_exp2(fmaf(x[cb][r], c, -m_ref[cb]));
                rs += p[r];
            }
            l_run[cb] += rs;
            pf[cb][0] = pack_frag(p, 0);
            pf[cb][1] = pack_frag(p, 8);
        }
        // P(u) and the prefetched fragments are consumed only by the next iteration; anchoring
        // them here keeps their instructions in this block, next to the matrix-core work
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) asm volatile("" : "+v"(pf[cb][0]), "+v"(pf[cb][1]), "+v"(l_run[cb]));
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) asm volatile("" : "+v"(ka[t8]));
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) asm volatile("" : "+v"(va[ks][db]));
    };

    issue(0, 0);
    dma_wait();
    __syncthreads();
    issue(min(1, nT - 1), 1);
    {   // scores of sub-tile 0 and the softmax reference of every query: its maximum there
        load_k(sm.k[0], 0);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[cb][r] = 0.f;
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) {
            s[0] = mma(ka[t8], qf_(0, t8), s[0]);
            s[1] = mma(ka[t8], qf_(1, t8), s[1]);
        }
        f32x16 x[2] = {s[0], s[1]};
        if (needs_mask(0, 0)) mask(x, 0, 0);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            float tm = x[cb][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) tm = fmaxf(tm, x[cb][r]);
            m_ref[cb] = partner_max(tm) * c;
        }
        load_k(sm.k[0], 32);      // K of sub-tile 1
        load_v(sm.v[0], 0);       // placeholder for "V of sub-tile -1": multiplied by P = 0
    }
    // Three LDS buffers, tile t in buffer t % 3.  The one barrier per tile opens the iteration
    // of the tile's first sub-tile: it publishes tile t+1 (read from this iteration on) and
    // retires tile t-1's buffer (its last fragments were fetched in the previous iteration),
    // which then receives tile t+2.
    int buf = 0;
    for (int t = 0; t < nT; ++t) {
        const int nbuf = buf + 1 == FWD_NBUF ? 0 : buf + 1;
        dma_wait();
        __syncthreads();
        issue(min(t + 2, nT - 1), nbuf + 1 == FWD_NBUF ? 0 : nbuf + 1);
        stage(2 * t, buf, nbuf);
        stage(2 * t + 1, buf, nbuf);
        buf = nbuf;
    }
    {   // drain: O^T += V^T P^T of the last sub-tile (its V fragments are already in registers)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                acc[db][0] = mma(va[ks][db], pf[0][ks], acc[db][0]);
                acc[db][1] = mma(va[ks][db], pf[1][ks], acc[db][1]);
            }
    }

    // normalise and store: lane holds, for its query, head elements 32db + 8(r/4) + 4g + r%4
    bool bad = false;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int qi = wrow0 + 32 * cb + lc;
        const float l_tot = l_run[cb] + partner(l_run[cb]);
        const float inv = 1.f / l_tot;
        float chk = 0.f;
        if (qi < S) {
            bf16_t* op = o + ((static_cast<size_t>(b) * S + qi) * Hq + h) * HD;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const float o0 = acc[db][cb][4 * r4] * inv, o1 = acc[db][cb][4 * r4 + 1] * inv,
                                o2 = acc[db][cb][4 * r4 + 2] * inv, o3 = acc[db][cb][4 * r4 + 3] * inv;
                    chk += (o0 + o1) + (o2 + o3);
                    u32x2 w = {pack_bf16x2(o0, o1), pack_bf16x2(o2, o3)};
                    *reinterpret_cast<u32x2*>(op + 32 * db + 8 * r4 + 4 * lg) = w;
                }
            if (lg == 0)
                lse[(static_cast<size_t>(b) * Hq + h) * S + qi] = (m_ref[cb] + fast_log2(l_tot)) * CART_LN2;
            // overflow of the fixed-reference softmax shows as a non-finite row sum or output
            bad |= !(l_tot < 3.0e38f) || !(fabsf(chk) < 3.0e38f);
        }
    }
    if (__any(bad) && lane == 0) sm_bad = 1;
    __syncthreads();
    if (threadIdx.x == 0) flags[blockIdx.x] = sm_bad;
}

// Recomputes the 256 queries of every flagged workgroup with a running-max loop on the vector
// ALU (one wavefront per query, lane l owns head elements 2l, 2l+1).  Launched after every
// forward call; a workgroup whose flag is clear returns at once.
__global__ __launch_bounds__(256) void attn_fwd_repair_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ zk, const bf16_t* __restrict__ zv, bf16_t* __restrict__ o,
    float* __restrict__ lse, const int* __restrict__ flags, int B, int S, int Hq, int Hkv, int P,
    float c) {
    if (flags[blockIdx.x] == 0) return;
    const int G = Hq / Hkv;
    const int nQt = (S + FWD_BM - 1) / FWD_BM;
    int id = blockIdx.x;
    const int hk = id % Hkv; id /= Hkv;
    const int g_ = id % G; id /= G;
    const int b = id % B; id /= B;
    const int qt = nQt - 1 - id;
    const int h = hk * G + g_;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    for (int i = qt * FWD_BM + wv; i < min(S, (qt + 1) * FWD_BM); i += 4) {
        const size_t row = (static_cast<size_t>(b) * S + i) * Hq + h;
        const uint32_t qw = *reinterpret_cast<const uint32_t*>(q + row * HD + 2 * lane);
        const float q0 = __uint_as_float(qw << 16), q1 = __uint_as_float(qw & 0xffff0000u);
        float m = -3.0e38f, l = 0.f, a0 = 0.f, a1 = 0.f;
        for (int j = 0; j < P + i + 1; ++j) {
            const size_t kr = j < P ? static_cast<size_t>(hk) * P + j
                                    : (static_cast<size_t>(b) * S + (j - P)) * Hkv + hk;
            const uint32_t kw = *reinterpret_cast<const uint32_t*>((j < P ? zk : k) + kr * HD + 2 * lane);
            const uint32_t vw = *reinterpret_cast<const uint32_t*>((j < P ? zv : v) + kr * HD + 2 * lane);
            const float sc = wave_sum(q0 * __uint_as_float(kw << 16) + q1 * __uint_as_float(kw & 0xffff0000u)) * c;
            const float nm = fmaxf(m, sc);
            const float corr = fast_exp2(m - nm), pj = fast_exp2(sc - nm);
            l = l * corr + pj;
            a0 = a0 * corr + pj * __uint_as_float(vw << 16);
            a1 = a1 * corr + pj * __uint_as_float(vw & 0xffff0000u);
            m = nm;
        }
        const float inv = 1.f / l;
        *reinterpret_cast<uint32_t*>(o + row * HD + 2 * lane) = pack_bf16x2(a0 * inv, a1 * inv);
        if (lane == 0) lse[(static_cast<size_t>(b) * Hq + h) * S + i] = (m + fast_log2(l)) * CART_LN2;
    }
}

bool attn_mfma_supported(const cart_attn_desc& d) {
    return d.dtype == CART_BF16 && d.D == 128;
}
static long fwd_grid(const cart_attn_desc& d) {
    return static_cast<long>((d.S + FWD_BM - 1) / FWD_BM) * d.B * d.Hq;
}
// one overflow flag per workgroup
size_t attn_mfma_fwd_workspace(const cart_attn_desc& d) {
    return (static_cast<size_t>(fwd_grid(d)) * sizeof(int) + 255) & ~static_cast<size_t>(255);
}

int launch_attn_fwd_mfma(const cart_attn_desc& d, float scale, const void* q, const void* k,
                         const void* v, const void* zk, const void* zv, void* o, float* lse,
                         void* ws, hipStream_t st) {
    const unsigned grid = static_cast<unsigned>(fwd_grid(d));
    int* flags = static_cast<int*>(ws);
    const bf16_t *Q = static_cast<const bf16_t*>(q), *K = static_cast<const bf16_t*>(k),
                 *V = static_cast<const bf16_t*>(v), *ZK = static_cast<const bf16_t*>(zk),
                 *ZV = static_cast<const bf16_t*>(zv);
    trace_begin(st);   // kernel order: forward, repair
    hipLaunchKernelGGL(attn_fwd_mfma_kernel, dim3(grid), dim3(256), 0, st, Q, K, V, ZK, ZV,
                       static_cast<bf16_t*>(o), lse, flags, d.B, d.S, d.Hq, d.Hkv, d.P, scale * CART_LOG2E);
    trace_mark(st);
    hipLaunchKernelGGL(attn_fwd_repair_kernel, dim3(grid), dim3(256), 0, st, Q, K, V, ZK, ZV,
                       static_cast<bf16_t*>(o), lse, flags, d.B, d.S, d.Hq, d.Hkv, d.P, scale * CART_LOG2E);
    trace_mark(st);
    return static_cast<int>(hipGetLastError());
}

}  // namespace cart
