// Cartridge attention backward on the matrix cores (bf16 in, fp32 accumulate, head_dim 128):
// the gradient of Eq. 1 over the cache of Sec. 3.2 with respect to Q, the own K/V and the
// trainable prefix Z (Sec. 3.2 trains Z by back-propagation with the model frozen).
//
// Three kernels, each with one 64-wide operand block held stationary in registers per wavefront
// and the other side streamed through LDS in tiles of 64 rows (sub-tiles of 32), in the same
// software pipeline as the forward kernel; the probabilities are recomputed from the saved
// log-sum-exp, so there is no running max and no rescale:
//   dq kernel   (queries stationary): S^T = K Q^T, dP^T = V dO^T, dQ^T += K^T dS^T
//   dk kernel   (keys stationary):    S = Q K^T,  dP = dO V^T,   dK^T += Q^T dS
//   dv kernel   (keys stationary):    S = Q K^T,                 dV^T += dO^T P
// with P = exp(scale S - lse), dS = P (dP - delta), delta_i = dO_i . O_i.  Nothing uses atomics:
// a key-stationary workgroup owns its keys' gradients for one sequence; prefix-slot gradients
// are written per sequence as fp32 partials and summed over the batch by dz_reduce_kernel in a
// fixed order, so results are bit-reproducible.
#include "attn_mfma.h"

namespace cart {
using namespace mfma;

constexpr int BWD_TILE = 64;                      // rows per LDS tile
constexpr int BWD_TILE_B = BWD_TILE * ROW_B;
constexpr int BWD_NBUF = 3;
constexpr int BWD_WG_ROWS = 256;                  // stationary rows per workgroup (4 x 64)

// ---- delta = rowsum(dO * O), lse2 = lse * log2(e); 16 lanes per row, 8 elements per lane ----
__global__ __launch_bounds__(256) void attn_bwd_prep_kernel(const bf16_t* __restrict__ o,
                                                            const bf16_t* __restrict__ d_o,
                                                            const float* __restrict__ lse,
                                                            float* __restrict__ delta,
                                                            float* __restrict__ lse2, int B, int S,
                                                            int Hq) {
    const long row = static_cast<long>(blockIdx.x) * 16 + (threadIdx.x >> 4);
    const long rows = static_cast<long>(B) * S * Hq;
    if (row >= rows) return;
    const int sub = threadIdx.x & 15;
    const u32x4 a = *reinterpret_cast<const u32x4*>(o + row * HD + sub * 8);
    const u32x4 g = *reinterpret_cast<const u32x4*>(d_o + row * HD + sub * 8);
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        s = fmaf(__uint_as_float(a[e] << 16), __uint_as_float(g[e] << 16), s);
        s = fmaf(__uint_as_float(a[e] & 0xffff0000u), __uint_as_float(g[e] & 0xffff0000u), s);
    }
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) s += __shfl_xor(s, off, 16);
    if (sub == 0) {
        const int h = row % Hq, i = (row / Hq) % S, b = row / (static_cast<long>(Hq) * S);
        const size_t st = (static_cast<size_t>(b) * Hq + h) * S + i;
        delta[st] = s;
        lse2[st] = lse[st] * CART_LOG2E;
    }
}

// store a transposed accumulator block set: lane owns output row `row_ptr` (nullptr: skip),
// register r of block db holds column 32 db + 8 (r/4) + 4 g + r%4
__device__ __forceinline__ void store_rows_bf16(const f32x16 (&acc)[4], bf16_t* row_ptr, int lg, float mul) {
    if (!row_ptr) return;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            u32x2 w = {pack_bf16x2(acc[db][4 * r4] * mul, acc[db][4 * r4 + 1] * mul),
                       pack_bf16x2(acc[db][4 * r4 + 2] * mul, acc[db][4 * r4 + 3] * mul)};
            *reinterpret_cast<u32x2*>(row_ptr + 32 * db + 8 * r4 + 4 * lg) = w;
        }
}
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_rows_f32(const f32x16 (&acc)[4], float* row_ptr, int lg, float mul) {
    if (!row_ptr) return;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            f32x4 w = {acc[db][4 * r4] * mul, acc[db][4 * r4 + 1] * mul, acc[db][4 * r4 + 2] * mul,
                       acc[db][4 * r4 + 3] * mul};
            *reinterpret_cast<f32x4*>(row_ptr + 32 * db + 8 * r4 + 4 * lg) = w;
        }
}

// =================================================================================================
// dQ: queries stationary
// =================================================================================================
// four buffers: the transposed K fragments of a tile's last sub-tile are fetched one iteration
// after the tile's other reads, so a tile's buffer is retired one tile later than in the other
// kernels
constexpr int DQ_NBUF = 4;
struct DqSmem {
    char k[DQ_NBUF][BWD_TILE_B];
    char v[DQ_NBUF][BWD_TILE_B];
};

__global__ __launch_bounds__(256, 1) void attn_bwd_dq_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ zk, const bf16_t* __restrict__ zv, const bf16_t* __restrict__ d_o,
    const float* __restrict__ lse2, const float* __restrict__ delta, bf16_t* __restrict__ dq, int B,
    int S, int Hq, int Hkv, int P, float c, float scale) {
    __shared__ DqSmem sm;
    const int G = Hq / Hkv;
    const int nQt = (S + BWD_WG_ROWS - 1) / BWD_WG_ROWS;
    int id = blockIdx.x;
    const int hk = id % Hkv; id /= Hkv;
    const int g_ = id % G; id /= G;
    const int b = id % B; id /= B;
    const int qt = nQt - 1 - id;
    const int h = hk * G + g_;
    const int lane = threadIdx.x & 63, lg = lane >> 5, lc = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q0 = qt * BWD_WG_ROWS, wrow0 = q0 + 64 * wv;

    u32x4 qf[2][8], gf[2][8];     // B operands: column = query, k = head element
    float l2[2], dl[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        int qi = wrow0 + 32 * cb + lc;
        qi = qi < S ? qi : S - 1;
        const size_t row = (static_cast<size_t>(b) * S + qi) * Hq + h;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            qf[cb][t] = *reinterpret_cast<const u32x4*>(q + row * HD + 8 * lg + 16 * t);
            gf[cb][t] = *reinterpret_cast<const u32x4*>(d_o + row * HD + 8 * lg + 16 * t);
        }
        const size_t st = (static_cast<size_t>(b) * Hq + h) * S + qi;
        l2[cb] = lse2[st];
        dl[cb] = delta[st];
    }
#define QF_(cb, t) __builtin_bit_cast(bf16x8, qf[cb][t])
#define GF_(cb, t) __builtin_bit_cast(bf16x8, gf[cb][t])

    const int nPt = (P + BWD_TILE - 1) / BWD_TILE;
    const int own_end = min(S, q0 + BWD_WG_ROWS);
    const int nT = nPt + (own_end + BWD_TILE - 1) / BWD_TILE;
    const char* zk_b = reinterpret_cast<const char*>(zk) + static_cast<size_t>(hk) * P * ROW_B;
    const char* zv_b = reinterpret_cast<const char*>(zv) + static_cast<size_t>(hk) * P * ROW_B;
    const size_t own_pitch = static_cast<size_t>(Hkv) * ROW_B;
    const char* k_b = reinterpret_cast<const char*>(k) + (static_cast<size_t>(b) * S * Hkv + hk) * ROW_B;
    const char* v_b = reinterpret_cast<const char*>(v) + (static_cast<size_t>(b) * S * Hkv + hk) * ROW_B;

    auto issue = [&](int t, int buf) __attribute__((always_inline)) {
        const bool pre = t < nPt;
        const int j0 = (pre ? t : t - nPt) * BWD_TILE;
        const int last = (pre ? P : S) - 1;
        const uint32_t pitch = pre ? static_cast<uint32_t>(ROW_B) : static_cast<uint32_t>(own_pitch);
        const char* kb = pre ? zk_b : k_b;
        const char* vb = pre ? zv_b : v_b;
        tile_load_async<BWD_TILE>(sm.k[buf], kb, j0, last, pitch);
        tile_load_async<BWD_TILE>(sm.v[buf], vb, j0, last, pitch);
    };

    f32x16 acc[4][2];   // dQ^T: [head-element block][query block]
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][cb][r] = 0.f;
    f32x16 s[2], dp[2];
    bf16x8 dsf[2][2];     // dS^T of sub-tile u-1 as B-operand fragments [query block][k-step]
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) dsf[cb][ks] = bf16x8{};

    auto needs_mask = [&](int t, int hb) __attribute__((always_inline)) {
        return t < nPt ? (t * BWD_TILE + 32 * hb + 32 > P) : ((t - nPt) * BWD_TILE + 32 * hb + 31 > wrow0);
    };
    auto mask = [&](f32x16 (&x)[2], int t, int hb) __attribute__((always_inline)) {
        const bool own = t >= nPt;
        const int j0 = (own ? t - nPt : t) * BWD_TILE + 32 * hb;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const int thr = (own ? wrow0 + 32 * cb + lc : P - 1) - j0 - 4 * lg;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (8 * (r >> 2) + (r & 3) > thr) x[cb][r] = NEG_BIG;
        }
    };
#ifndef CART_DQ_PIN_Q
#define CART_DQ_PIN_Q 1
#endif
#ifndef CART_DQ_PREFETCH_V
#define CART_DQ_PREFETCH_V 0
#endif
    auto pin = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
#if CART_DQ_PIN_Q
                asm volatile("" : "+a"(qf[cb][t]));
#endif
            }
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) asm volatile("" : "+a"(acc[db][cb]));
    };
    // row-wise K (and V) fragments of sub-tile u+1 are fetched one iteration ahead (loop-carried)
    bf16x8 ka[8], va[8];
    auto load_nat = [&](int buf, int r0, bool with_v) __attribute__((always_inline)) {
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) {
            ka[t8] = lds_frag_n(sm.k[0] + buf * BWD_TILE_B, r0 + lc, 16 * t8 + 8 * lg);
            if (with_v) va[t8] = lds_frag_n(sm.v[0] + buf * BWD_TILE_B, r0 + lc, 16 * t8 + 8 * lg);
        }
    };
    auto scores = [&](int vbuf, int vr0) __attribute__((always_inline)) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[cb][r] = 0.f; dp[cb][r] = 0.f; }
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) {
            s[0] = mma(ka[t8], QF_(0, t8), s[0]);
            s[1] = mma(ka[t8], QF_(1, t8), s[1]);
#if CART_DQ_PREFETCH_V
            const bf16x8 a2 = va[t8];
#else
            const bf16x8 a2 = lds_frag_n(sm.v[0] + vbuf * BWD_TILE_B, vr0 + lc, 16 * t8 + 8 * lg);
#endif
            dp[0] = mma(a2, GF_(0, t8), dp[0]);
            dp[1] = mma(a2, GF_(1, t8), dp[1]);
        }
    };
    // Iteration u (sub-tile hb of tile t in buffer buf; nbuf holds tile t+1).  On entry: s, dp =
    // scores of sub-tile u; ka (va) = row-wise fragments of sub-tile u+1; dsf = dS^T(u-1).
    auto stage = [&](int t, int hb, int buf, int nbuf) __attribute__((always_inline)) {
        f32x16 x[2] = {s[0], s[1]};
        f32x16 y[2] = {dp[0], dp[1]};
        if (needs_mask(t, hb)) mask(x, t, hb);
        pin();
        // matrix cores: scores of sub-tile u+1, dQ^T += K^T(u-1) dS^T(u-1)
        scores(hb ? nbuf : buf, hb ? 0 : 32);
        // (the very first iteration has no predecessor: it multiplies tile 0 by dS = 0)
        const char* kt_prev = sm.k[0] + ((hb || t == 0) ? buf : ((buf + DQ_NBUF - 1) & (DQ_NBUF - 1))) * BWD_TILE_B;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const bf16x8 a = lds_frag_t(kt_prev, (hb ? 0 : 32) + 16 * ks, 32 * db, lane);
                acc[db][0] = mma(a, dsf[0][ks], acc[db][0]);
                acc[db][1] = mma(a, dsf[1][ks], acc[db][1]);
            }
        // row-wise fragments of sub-tile u+2
        load_nat(nbuf, 32 * hb, CART_DQ_PREFETCH_V);
        // vector ALU: dS^T of sub-tile u
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            f32x16 w;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = fast_exp2(fmaf(x[cb][r], c, -l2[cb]));
                w[r] = p * (y[cb][r] - dl[cb]);
            }
            dsf[cb][0] = pack_frag(w, 0);
            dsf[cb][1] = pack_frag(w, 8);
        }
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) asm volatile("" : "+v"(dsf[cb][0]), "+v"(dsf[cb][1]));
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) {
            asm volatile("" : "+v"(ka[t8]));
#if CART_DQ_PREFETCH_V
            asm volatile("" : "+v"(va[t8]));
#endif
        }
    };

    issue(0, 0);
    dma_wait();
    __syncthreads();
    issue(min(1, nT - 1), 1);
    pin();
    load_nat(0, 0, CART_DQ_PREFETCH_V);
    scores(0, 0);                          // sub-tile 0
    load_nat(0, 32, CART_DQ_PREFETCH_V);   // sub-tile 1
    // Tile t lives in buffer t % 4.  The one barrier per tile opens the iteration of the tile's
    // first sub-tile: it publishes tile t+1 and retires tile t-2's buffer (tile t-1's transposed
    // K is still read in this iteration), which then receives tile t+2.
    int buf = 0;
    for (int t = 0; t < nT; ++t) {
        const int nbuf = (buf + 1) & (DQ_NBUF - 1);
        dma_wait();
        __syncthreads();
        issue(min(t + 2, nT - 1), (buf + 2) & (DQ_NBUF - 1));
        stage(t, 0, buf, nbuf);
        stage(t, 1, buf, nbuf);
        buf = nbuf;
    }
    {   // drain: dQ^T += K^T dS^T of the last sub-tile
        const char* kt_prev = sm.k[0] + ((buf + DQ_NBUF - 1) & (DQ_NBUF - 1)) * BWD_TILE_B;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const bf16x8 a = lds_frag_t(kt_prev, 32 + 16 * ks, 32 * db, lane);
                acc[db][0] = mma(a, dsf[0][ks], acc[db][0]);
                acc[db][1] = mma(a, dsf[1][ks], acc[db][1]);
            }
    }
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int qi = wrow0 + 32 * cb + lc;
        f32x16 col[4] = {acc[0][cb], acc[1][cb], acc[2][cb], acc[3][cb]};
        store_rows_bf16(col, qi < S ? dq + ((static_cast<size_t>(b) * S + qi) * Hq + h) * HD : nullptr, lg, scale);
    }
}

// =================================================================================================
// dK / dV: keys stationary
// =================================================================================================
// The dV kernel fetches every LDS fragment one iteration ahead and needs three tile buffers.  The
// dK kernel holds twice the stationary fragments (K and V) and twice the score accumulators, has
// no registers left for prefetched fragments, reads them where used, and therefore retires a
// tile's buffer one tile later: four buffers.
template <int NBUF>
struct KsSmem {
    char q[NBUF][BWD_TILE_B];
    char g[NBUF][BWD_TILE_B];
    float l2[NBUF][BWD_TILE];
    float dl[NBUF][BWD_TILE];
};

// One workgroup = 256 keys of one (sequence, KV head): a block of prefix slots, or a block of the
// sequence's own tokens.  It streams the queries that see those keys: all tokens of all heads of
// the group for prefix slots, tokens at or after the block for own keys.
template <bool IS_DK>
__global__ __launch_bounds__(256, 1) void attn_bwd_kstat_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ zk, const bf16_t* __restrict__ zv, const bf16_t* __restrict__ d_o,
    const float* __restrict__ lse2, const float* __restrict__ delta, bf16_t* __restrict__ out_own,
    float* __restrict__ part, int B, int S, int Hq, int Hkv, int P, float c, float scale) {
    constexpr int NBUF = IS_DK ? 4 : 3;
    constexpr bool PREFETCH = !IS_DK;
    __shared__ KsSmem<NBUF> sm;
    const int G = Hq / Hkv;
    const int nPb = (P + BWD_WG_ROWS - 1) / BWD_WG_ROWS, nOb = (S + BWD_WG_ROWS - 1) / BWD_WG_ROWS;
    const int nKb = nPb + nOb;
    int id = blockIdx.x;
    const int hk = id % Hkv; id /= Hkv;
    const int kb = id % nKb;
    const int b = id / nKb;
    const bool pre = kb < nPb;
    const int key0 = (pre ? kb : kb - nPb) * BWD_WG_ROWS;
    const int nkeys = pre ? P : S;
    const int lane = threadIdx.x & 63, lg = lane >> 5, lc = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wkey0 = key0 + 64 * wv;

    // this wavefront's 64 keys as B operands: column = key, k = head element
    u32x4 kf[2][8], vf[2][8];
#pragma unroll
    for (int kc = 0; kc < 2; ++kc) {
        const int key = min(wkey0 + 32 * kc + lc, nkeys - 1);
        const size_t row = pre ? static_cast<size_t>(hk) * P + key
                               : (static_cast<size_t>(b) * S + key) * Hkv + hk;
        const bf16_t* kp = (pre ? zk : k) + row * HD + 8 * lg;
        const bf16_t* vp = (pre ? zv : v) + row * HD + 8 * lg;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            kf[kc][t] = *reinterpret_cast<const u32x4*>(kp + 16 * t);
            if (IS_DK) vf[kc][t] = *reinterpret_cast<const u32x4*>(vp + 16 * t);
        }
    }

    const int nQtAll = (S + BWD_TILE - 1) / BWD_TILE;
    const int qt0 = pre ? 0 : key0 / BWD_TILE;
    const int nq = nQtAll - qt0;
    const int nT = G * nq;            // query tiles streamed: head-major, token tiles inside
    const char* q_c = reinterpret_cast<const char*>(q);
    const char* g_c = reinterpret_cast<const char*>(d_o);
    const size_t q_pitch = static_cast<size_t>(Hq) * ROW_B;

    auto issue = [&](int T, int buf) __attribute__((always_inline)) {
        const int gi = T / nq, qt = qt0 + T - gi * nq;
        const int h = hk * G + gi;
        const int i0 = qt * BWD_TILE;
        const size_t base = (static_cast<size_t>(b) * S * Hq + h) * ROW_B;
        tile_load_async<BWD_TILE>(sm.q[buf], q_c + base, i0, S - 1, static_cast<uint32_t>(q_pitch));
        tile_load_async<BWD_TILE>(sm.g[buf], g_c + base, i0, S - 1, static_cast<uint32_t>(q_pitch));
        // the tile's 64 lse2 / delta values: one 4-byte direct-to-LDS load per lane
        if (wv < 2) {
            const float* src = (wv == 0 ? lse2 : delta) + (static_cast<size_t>(b) * Hq + h) * S;
            float* dst = wv == 0 ? sm.l2[buf] : sm.dl[buf];
            dma4(reinterpret_cast<const char*>(src), static_cast<uint32_t>(min(i0 + lane, S - 1)) * 4u, lds_addr(dst));
        }
    };
    auto tile_i0 = [&](int T) __attribute__((always_inline)) {
        const int gi = T / nq;
        return (qt0 + T - gi * nq) * BWD_TILE;
    };

    f32x16 acc[4][2];   // dK^T or dV^T: [head-element block][key block]
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][kc][r] = 0.f;
    f32x16 s[2], dp[2];   // [key block]: rows = 32 queries of the sub-tile, one iteration ahead
    bf16x8 xf[2][2];      // P or dS of sub-tile u-1 as B-operand fragments [key block][k-step]
#pragma unroll
    for (int kc = 0; kc < 2; ++kc)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) xf[kc][ks] = bf16x8{};

    // a query row of the sub-tile is hidden from a key when it precedes it (own keys) or lies
    // past the end of the sequence (clamped tile rows)
    auto needs_mask = [&](int T, int hb) __attribute__((always_inline)) {
        const int i0 = tile_i0(T) + 32 * hb;
        return (!pre && i0 < wkey0 + 63) || (i0 + 32 > S);
    };
    auto mask = [&](f32x16 (&x)[2], int T, int hb) __attribute__((always_inline)) {
        const int i0 = tile_i0(T) + 32 * hb;
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) {
            // row i0 + d_row(r, lg) is visible iff it is >= the lane's key (own) and < S
            const int lo = (pre ? 0 : wkey0 + 32 * kc + lc) - i0 - 4 * lg;
            const int hi = S - i0 - 4 * lg;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rr = 8 * (r >> 2) + (r & 3);
                if (rr < lo || rr >= hi) x[kc][r] = NEG_BIG;
            }
        }
    };
    // the stationary fragments live in accumulation registers (read directly as B operands)
    constexpr bool PIN_K = true;
    auto pin = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
            for (int t = 0; t < 8; ++t)
                if (PIN_K) asm volatile("" : "+a"(kf[kc][t]));
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int kc = 0; kc < 2; ++kc) asm volatile("" : "+a"(acc[db][kc]));
    };
#define KF_(kc, t) __builtin_bit_cast(bf16x8, kf[kc][t])
#define VF_(kc, t) __builtin_bit_cast(bf16x8, vf[kc][t])

    // LDS -> register fragments run one iteration ahead of their use (loop-carried): row-wise Q
    // (and dO) of sub-tile u+1, transposed dO (or Q) of sub-tile u-1
    bf16x8 qa[8], ta[2][4];
    auto load_nat = [&](int buf, int r0) __attribute__((always_inline)) {
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) {
            qa[t8] = lds_frag_n(sm.q[0] + buf * BWD_TILE_B, r0 + lc, 16 * t8 + 8 * lg);
        }
    };
    auto load_tr = [&](int buf, int r0) __attribute__((always_inline)) {
        const char* at = (IS_DK ? sm.q[0] : sm.g[0]) + buf * BWD_TILE_B;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) ta[ks][db] = lds_frag_t(at, r0 + 16 * ks, 32 * db, lane);
    };
    // scores of one sub-tile: from the prefetched fragments, or (dK) straight from LDS buffer
    // nb, rows r0..
    auto scores = [&](int nb, int r0) __attribute__((always_inline)) {
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[kc][r] = 0.f; if (IS_DK) dp[kc][r] = 0.f; }
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) {
            const bf16x8 a = PREFETCH ? qa[t8] : lds_frag_n(sm.q[0] + nb * BWD_TILE_B, r0 + lc, 16 * t8 + 8 * lg);
            s[0] = mma(a, KF_(0, t8), s[0]);
            s[1] = mma(a, KF_(1, t8), s[1]);
            if (IS_DK) {
                const bf16x8 a2 = lds_frag_n(sm.g[0] + nb * BWD_TILE_B, r0 + lc, 16 * t8 + 8 * lg);
                dp[0] = mma(a2, VF_(0, t8), dp[0]);
                dp[1] = mma(a2, VF_(1, t8), dp[1]);
            }
        }
    };
    // Iteration u (sub-tile hb of streamed tile T, in LDS buffer buf; nbuf holds tile T+1).  On
    // entry: s (dp) = scores of sub-tile u, qa (ga) = row-wise fragments of sub-tile u+1,
    // ta = transposed fragments of sub-tile u-1, xf = P / dS of sub-tile u-1.
    auto stage = [&](int T, int hb, int buf, int nbuf) __attribute__((always_inline)) {
        // scores of sub-tile u move to ordinary registers (their accumulators are reused); the
        // rare masked sub-tile is patched here, outside the main block
        f32x16 x[2] = {s[0], s[1]};
        f32x16 y[2];
        if (IS_DK) { y[0] = dp[0]; y[1] = dp[1]; }
        if (needs_mask(T, hb)) mask(x, T, hb);
        pin();
        scores(hb ? nbuf : buf, hb ? 0 : 32);
        // (dK: transposed fragments of sub-tile u-1 read here; the very first iteration has no
        // predecessor and multiplies tile 0 by xf = 0)
        if (!PREFETCH) load_tr((hb || T == 0) ? buf : (buf + NBUF - 1) % NBUF, hb ? 0 : 32);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                acc[db][0] = mma(ta[ks][db], xf[0][ks], acc[db][0]);
                acc[db][1] = mma(ta[ks][db], xf[1][ks], acc[db][1]);
            }
        // fragments for the next iteration: row-wise of sub-tile u+2, transposed of sub-tile u
        if (PREFETCH) {
            load_nat(nbuf, 32 * hb);
            load_tr(buf, 32 * hb);
        }
        // per-row lse2 / delta of this sub-tile (rows 8 j + 4 g + (0..3)) are read from LDS four
        // rows at a time, right where they are used
        f32x16 w[2];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const f32x4 lr = *reinterpret_cast<const f32x4*>(&sm.l2[buf][32 * hb + 8 * j + 4 * lg]);
            f32x4 dr = {0.f, 0.f, 0.f, 0.f};
            if (IS_DK) dr = *reinterpret_cast<const f32x4*>(&sm.dl[buf][32 * hb + 8 * j + 4 * lg]);
#pragma unroll
            for (int kc = 0; kc < 2; ++kc)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = 4 * j + e;
                    const float p = fast_exp2(fmaf(x[kc][r], c, -lr[e]));
                    w[kc][r] = IS_DK ? p * (y[kc][r] - dr[e]) : p;
                }
        }
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) {
            xf[kc][0] = pack_frag(w[kc], 0);
            xf[kc][1] = pack_frag(w[kc], 8);
        }
        // consumed only by the next iteration: anchored here so that their instructions stay in
        // this block, next to the matrix-core work
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) asm volatile("" : "+v"(xf[kc][0]), "+v"(xf[kc][1]));
        if (PREFETCH) {
#pragma unroll
            for (int t8 = 0; t8 < 8; ++t8) asm volatile("" : "+v"(qa[t8]));
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int db = 0; db < 4; ++db) asm volatile("" : "+v"(ta[ks][db]));
        }
    };

    issue(0, 0);
    dma_wait();
    __syncthreads();
    issue(min(1, nT - 1), 1);
    pin();
    if (PREFETCH) load_nat(0, 0);
    scores(0, 0);             // sub-tile 0
    if (PREFETCH) {
        load_nat(0, 32);      // row-wise fragments of sub-tile 1
        load_tr(0, 0);        // placeholder for "sub-tile -1": multiplied by xf = 0
    }
    // Streamed tile T lives in buffer T % NBUF.  The one barrier per tile opens the iteration of
    // the tile's first sub-tile: it publishes tile T+1 and retires the buffer of the oldest tile
    // no longer read (T-1 with prefetched fragments, T-2 without), which receives tile T+2.
    int buf = 0;
    for (int T = 0; T < nT; ++T) {
        const int nbuf = (buf + 1) % NBUF;
        dma_wait();
        __syncthreads();
        issue(min(T + 2, nT - 1), (buf + 2) % NBUF);
        stage(T, 0, buf, nbuf);
        stage(T, 1, buf, nbuf);
        buf = nbuf;
    }
    if (!PREFETCH) load_tr((buf + NBUF - 1) % NBUF, 32);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)      // drain: the last sub-tile's contribution
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            acc[db][0] = mma(ta[ks][db], xf[0][ks], acc[db][0]);
            acc[db][1] = mma(ta[ks][db], xf[1][ks], acc[db][1]);
        }
    const float mul = IS_DK ? scale : 1.f;
#pragma unroll
    for (int kc = 0; kc < 2; ++kc) {
        const int key = wkey0 + 32 * kc + lc;
        f32x16 col[4] = {acc[0][kc], acc[1][kc], acc[2][kc], acc[3][kc]};
        if (pre)
            store_rows_f32(col, key < P ? part + ((static_cast<size_t>(b) * Hkv + hk) * P + key) * HD : nullptr, lg, mul);
        else
            store_rows_bf16(col, key < S ? out_own + ((static_cast<size_t>(b) * S + key) * Hkv + hk) * HD : nullptr, lg, mul);
    }
}

// dZ[hk,slot,:] = sum_b part[b,hk,slot,:] in order of b (+ the previous value when accumulating);
// rows below n_frozen are 0 / left alone.  One 16-byte vector per thread.
__global__ __launch_bounds__(256) void dz_reduce_kernel(const float* __restrict__ part,
                                                        float* __restrict__ dz, int B, long n4,
                                                        int P, int n_frozen, int accumulate) {
    const long i = static_cast<long>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n4) return;
    const int slot = (i / (HD / 4)) % P;
    const f32x4* src = reinterpret_cast<const f32x4*>(part);
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    if (slot >= n_frozen)
        for (int b = 0; b < B; ++b) a += src[static_cast<long>(b) * n4 + i];
    f32x4* dst = reinterpret_cast<f32x4*>(dz);
    if (accumulate) a += dst[i];
    dst[i] = a;
}

bool attn_mfma_bwd_supported(const cart_attn_desc& d) { return d.dtype == CART_BF16 && d.D == 128; }

static size_t r256(size_t n) { return (n + 255) & ~static_cast<size_t>(255); }

// beyond the delta array: lse2 [B,Hq,S] and the two per-sequence dZ partial buffers [B,Hkv,P,128]
size_t attn_mfma_bwd_workspace(const cart_attn_desc& d) {
    const size_t rows = r256(static_cast<size_t>(d.B) * d.Hq * d.S * sizeof(float));
    const size_t part = r256(static_cast<size_t>(d.B) * d.Hkv * d.P * HD * sizeof(float));
    return rows + 2 * part;
}

int launch_attn_bwd_mfma(const cart_attn_desc& d, float scale, const void* q, const void* k,
                         const void* v, const void* zk, const void* zv, const void* o,
                         const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                         float* dzk, float* dzv, void* ws, hipStream_t st) {
    const size_t rows_b = r256(static_cast<size_t>(d.B) * d.Hq * d.S * sizeof(float));
    const size_t part_b = r256(static_cast<size_t>(d.B) * d.Hkv * d.P * HD * sizeof(float));
    char* w = static_cast<char*>(ws);
    float* delta = reinterpret_cast<float*>(w);
    float* lse2 = reinterpret_cast<float*>(w + rows_b);
    float* part_k = reinterpret_cast<float*>(w + 2 * rows_b);
    float* part_v = reinterpret_cast<float*>(w + 2 * rows_b + part_b);
    const bf16_t *Q = static_cast<const bf16_t*>(q), *K = static_cast<const bf16_t*>(k),
                 *V = static_cast<const bf16_t*>(v), *ZK = static_cast<const bf16_t*>(zk),
                 *ZV = static_cast<const bf16_t*>(zv), *DO = static_cast<const bf16_t*>(d_o);
    const float c = scale * CART_LOG2E;
    const long rows = static_cast<long>(d.B) * d.S * d.Hq;
    trace_begin(st);   // kernel order: prep, dq, dk, dv, dz reduce (k, v)
    hipLaunchKernelGGL(attn_bwd_prep_kernel, dim3(static_cast<unsigned>((rows + 15) / 16)), dim3(256), 0, st,
                       static_cast<const bf16_t*>(o), DO, lse, delta, lse2, d.B, d.S, d.Hq);
    trace_mark(st);
    const int nQt = (d.S + BWD_WG_ROWS - 1) / BWD_WG_ROWS;
    hipLaunchKernelGGL(attn_bwd_dq_kernel, dim3(static_cast<unsigned>(static_cast<long>(nQt) * d.B * d.Hq)), dim3(256),
                       0, st, Q, K, V, ZK, ZV, DO, lse2, delta, static_cast<bf16_t*>(dq), d.B, d.S, d.Hq,
                       d.Hkv, d.P, c, scale);
    trace_mark(st);
    const int nKb = (d.P + BWD_WG_ROWS - 1) / BWD_WG_ROWS + (d.S + BWD_WG_ROWS - 1) / BWD_WG_ROWS;
    const unsigned kgrid = static_cast<unsigned>(static_cast<long>(nKb) * d.B * d.Hkv);
    hipLaunchKernelGGL(attn_bwd_kstat_kernel<true>, dim3(kgrid), dim3(256), 0, st, Q, K, V, ZK, ZV, DO, lse2,
                       delta, static_cast<bf16_t*>(dk), part_k, d.B, d.S, d.Hq, d.Hkv, d.P, c, scale);
    trace_mark(st);
    hipLaunchKernelGGL(attn_bwd_kstat_kernel<false>, dim3(kgrid), dim3(256), 0, st, Q, K, V, ZK, ZV, DO, lse2,
                       delta, static_cast<bf16_t*>(dv), part_v, d.B, d.S, d.Hq, d.Hkv, d.P, c, scale);
    trace_mark(st);
    if (d.P > 0) {
        const long n4 = static_cast<long>(d.Hkv) * d.P * HD / 4;
        const unsigned rg = static_cast<unsigned>((n4 + 255) / 256);
        hipLaunchKernelGGL(dz_reduce_kernel, dim3(rg), dim3(256), 0, st, part_k, dzk, d.B, n4, d.P, d.n_frozen, d.dz_accumulate);
        hipLaunchKernelGGL(dz_reduce_kernel, dim3(rg), dim3(256), 0, st, part_v, dzv, d.B, n4, d.P, d.n_frozen, d.dz_accumulate);
        trace_mark(st);
    }
    return static_cast<int>(hipGetLastError());
}

}  // namespace cart
