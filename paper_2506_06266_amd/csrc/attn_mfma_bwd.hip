// Cartridge attention backward on the matrix cores (bf16 in, fp32 accumulate, head_dim 128):
// the gradient of Eq. 1 over the cache of Sec. 3.2 with respect to Q, the own K/V and the
// trainable prefix Z (Sec. 3.2 trains Z by back-propagation with the model frozen).
//
// This file: the dQ kernel (queries stationary: S^T = K Q^T, dP^T = V dO^T, dQ^T += K^T dS^T, with
// P = exp(scale S - lse), dS = P (dP - delta), delta_i = dO_i . O_i formed in its prologue and
// written out for the key-side kernel), the fixed-order reduction of the prefix-gradient partials,
// and the launcher of the whole backward call.  dK, dV and the partials of dZ come from the
// key-stationary kernel of attn_mfma_bwd_kv.hip.  The probabilities are recomputed from the saved
// log-sum-exp, so there is no running max and no rescale; nothing uses atomics, so results are
// bit-reproducible.
#include "attn_mfma.h"

namespace cart {
using namespace mfma;

// 1: fold c = softmax_scale * log2(e) into the register-resident operand (one extra bf16
// rounding) and -lse2 into the score product's init value.  0: scale in fp32,
// P = 2^fma(score, c, -lse2): exact, one more vector-ALU instruction per element in dK / dV.
#ifndef CART_PRESCALE
#define CART_PRESCALE 0
#endif

constexpr int BWD_TILE = 64;                      // rows per LDS tile
constexpr int BWD_TILE_B = BWD_TILE * ROW_B;
constexpr int BWD_WG_ROWS = 256;                  // stationary rows per workgroup (4 x 64)
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

// =================================================================================================
// dQ: queries stationary
// =================================================================================================
// One workgroup = 256 consecutive queries of one (sequence, query head); each wavefront keeps its
// 64 queries' Q (scaled by c = softmax_scale * log2(e)) and dO as B-operand fragments in
// accumulation registers, next to the dQ^T accumulators.  Key tiles (K and V rows) stream through
// LDS in the forward kernel's order: first the tiles every query sees entirely, through a loop
// without masking code, then the ragged prefix tile and the diagonal tiles through a copy that
// masks.  Per sub-tile of 32 keys:
//   S^T = K Q^T, dP^T = V dO^T,  dS^T = 2^(S^T - lse2) (dP^T - delta),  dQ^T += K^T dS^T.
// The iteration is laid out like the dK kernel's: 48 fenced groups; the scores / dP of query
// block 1 live in one register set, those of block 0 in two used alternately; the transposed K
// fragments of the previous sub-tile are fetched about ten groups ahead, so a tile is read over
// three tile iterations: four buffers.
constexpr int DQ_NBUF = 4;
struct DqSmem {
    struct { char k[BWD_TILE_B]; char v[BWD_TILE_B]; } t[DQ_NBUF];
};

__global__ __launch_bounds__(256, 1) void attn_bwd_dq_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ zk, const bf16_t* __restrict__ zv, const bf16_t* __restrict__ o,
    const bf16_t* __restrict__ d_o, const float* __restrict__ lse, float* __restrict__ nlse2,
    float* __restrict__ ndelta, bf16_t* __restrict__ dq, const int32_t* __restrict__ cu,
    const int32_t* __restrict__ row_lo, int n_tok, int B, int Smax, int Hq, int Hkv, int P, float c, float scale) {
    constexpr int NBUF = DQ_NBUF;
    constexpr int BUF_B = 2 * BWD_TILE_B;
    constexpr int V_OFF = BWD_TILE_B;
    __shared__ DqSmem sm;
    const int G = Hq / Hkv;
    const int nQt = (Smax + BWD_WG_ROWS - 1) / BWD_WG_ROWS;
    int id = blockIdx.x;
    const int hk = id % Hkv; id /= Hkv;
    const int g_ = id % G; id /= G;
    const int qt = nQt - 1 - id % nQt;
    const int b = id / nQt;
    const int h = hk * G + g_;
    const int lane = threadIdx.x & 63, lg = lane >> 5, lc = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q0 = qt * BWD_WG_ROWS, wrow0 = q0 + 64 * wv;
    // packed layout: the grid covers the longest sequence; nothing to do past the end of this one.
    // With row_lo (B = 1, S = all packed rows) the query tiles are cut from the packed rows as in
    // the forward kernel and row i sees the own keys row_lo[i] .. i.
    const SeqSpan sp = seq_span(cu, b, n_tok, Smax, Hq);
    const int S = sp.len;
    const size_t t0 = sp.t0;
    if (q0 >= S) return;

    // The row statistics of the backward pass are formed here, where O and dO of every query row
    // pass through registers anyway: -delta = -rowsum(dO * O) and -lse2 = -lse * log2(e)
    // (negated: they enter the products as init values).  They are also written out for the dK
    // and dV kernels, which run after this one.
    u32x4 qf[2][8], gf[2][8];     // B operands: column = query, k = head element
    float nl2[2], ndl[2];         // -lse2, -delta of the lane's queries
    int lo_q[2] = {0, 0};         // first own key the lane's queries see
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int qi_raw = wrow0 + 32 * cb + lc;
        const int qi = qi_raw < S ? qi_raw : S - 1;
        if (row_lo) lo_q[cb] = row_lo[qi];
        const size_t row = (t0 + qi) * Hq + h;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const u32x4 w = *reinterpret_cast<const u32x4*>(q + row * HD + 8 * lg + 16 * t);
#if CART_PRESCALE
#pragma unroll
            for (int i = 0; i < 4; ++i)
                qf[cb][t][i] = pack_bf16x2(__uint_as_float(w[i] << 16) * c, __uint_as_float(w[i] & 0xffff0000u) * c);
#else
            qf[cb][t] = w;
#endif
            gf[cb][t] = *reinterpret_cast<const u32x4*>(d_o + row * HD + 8 * lg + 16 * t);
        }
        float ds = 0.f;       // the lane's half of the row's head elements, the partner lane's added below
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const u32x4 ow = *reinterpret_cast<const u32x4*>(o + row * HD + 8 * lg + 16 * t);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ds = fmaf(__uint_as_float(ow[i] << 16), __uint_as_float(gf[cb][t][i] << 16), ds);
                ds = fmaf(__uint_as_float(ow[i] & 0xffff0000u), __uint_as_float(gf[cb][t][i] & 0xffff0000u), ds);
            }
        }
        ds += partner(ds);
        nl2[cb] = -lse[sp.stat_b + h * sp.stat_h + qi] * CART_LOG2E;
        ndl[cb] = -ds;
        if (lg == 0 && qi_raw < S) {      // internal layout [Hq][all token rows], both input layouts
            const size_t st = static_cast<size_t>(h) * n_tok + t0 + qi;
            nlse2[st] = nl2[cb];
            ndelta[st] = ndl[cb];
        }
    }
    // -delta of the lane's queries in all 16 registers of a set: the dP^T products start from it
    // (their init value), so that dP^T - delta needs no instruction of its own
    f32x16 ndi[2];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) ndi[cb][r] = ndl[cb];
    f32x16 acc[4][2];   // dQ^T: [head-element block][query block]
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][cb][r] = 0.f;
    auto pin = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                asm volatile("" : "+a"(qf[cb][t]));
                asm volatile("" : "+a"(gf[cb][t]));
            }
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) asm volatile("" : "+a"(acc[db][cb]));
    };
    pin();

    // tile order: see the forward kernel
    const int nPf = P / BWD_TILE;
    const int rag = (P % BWD_TILE) ? 1 : 0;
    const int own_end = min(S, q0 + BWD_WG_ROWS);
    const int lo_first = row_lo ? row_lo[q0] : 0, lo_last = row_lo ? row_lo[own_end - 1] : 0;
    const int tA = lo_first / BWD_TILE, tU0 = (lo_last + BWD_TILE - 1) / BWD_TILE, tD = q0 / BWD_TILE;
    const int nOf = max(0, tD - tU0);
    const int nLow = min(tU0, tD) - tA;
    const int nMain = nPf + nOf;
    const int nT = nMain + rag + nLow + (own_end + BWD_TILE - 1) / BWD_TILE - tD;
    const char* zk_b = reinterpret_cast<const char*>(zk) + static_cast<size_t>(hk) * P * ROW_B;
    const char* zv_b = reinterpret_cast<const char*>(zv) + static_cast<size_t>(hk) * P * ROW_B;
    const uint32_t own_pitch = static_cast<uint32_t>(Hkv) * ROW_B;
    const char* k_b = reinterpret_cast<const char*>(k) + (t0 * Hkv + hk) * ROW_B;
    const char* v_b = reinterpret_cast<const char*>(v) + (t0 * Hkv + hk) * ROW_B;
    auto tile_pre = [&](int t) __attribute__((always_inline)) { return t < nPf || (rag && t == nMain); };
    auto tile_j0 = [&](int t) __attribute__((always_inline)) {
        const int m = t - nMain - rag;
        return (t < nPf ? t : t < nMain ? tU0 + t - nPf : (rag && t == nMain) ? nPf : m < nLow ? tA + m : tD + m - nLow) * BWD_TILE;
    };
    const uint32_t dma_c0 = (lane & 15) ^ (((lane >> 4) & 3) << 2);
    struct TileSrc { const char* kb; const char* vb; int lim; uint32_t pitch; uint32_t lds_k, lds_v; };
    auto tile_src = [&](int t, int buf) __attribute__((always_inline)) {
        const bool pre = tile_pre(t);
        const int j0 = tile_j0(t);
        TileSrc ts;
        ts.pitch = pre ? static_cast<uint32_t>(ROW_B) : own_pitch;
        ts.kb = (pre ? zk_b : k_b) + static_cast<size_t>(j0) * ts.pitch;
        ts.vb = (pre ? zv_b : v_b) + static_cast<size_t>(j0) * ts.pitch;
        ts.lim = (pre ? P : S) - 1 - j0;
        ts.lds_k = lds_addr(sm.t[buf].k);
        ts.lds_v = lds_addr(sm.t[buf].v);
        return ts;
    };
    auto dma_piece = [&](const TileSrc& ts, int n) __attribute__((always_inline)) {
        const int i = n & 3;
        const int r0 = (4 * wv + i) * 4;
        const uint32_t voff = __umul24(min(r0 + (lane >> 4), ts.lim), ts.pitch) + ((dma_c0 ^ i) << 4);
        if (n < 4) dma16(ts.kb, voff, ts.lds_k + r0 * ROW_B);
        else       dma16(ts.vb, voff, ts.lds_v + r0 * ROW_B);
    };
    // hidden entries of query block cb in the scores of the sub-tile whose first key is j0
    auto mask1 = [&](f32x16& x, int cb, bool pre, int j0) __attribute__((always_inline)) {
        mask_above(x, (pre ? P - 1 : wrow0 + 32 * cb + lc) - j0 - 4 * lg);
        if (row_lo && !pre) mask_below(x, lo_q[cb] - j0 - 4 * lg);
    };

    // per-lane LDS addresses: row-wise K fragments (V: + V_OFF) of the tile of sub-tile u+1,
    // transposed K fragments of the tile of sub-tile u-1 (they follow half a tile iteration later)
    uint32_t kofs[8], tofs[4][2];
    {
        const uint32_t t0 = lds_addr(sm.t[0].k);
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) kofs[t8] = t0 + frag_n_ofs(lane, t8);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            frag_t_ofs(lane, db, tofs[db][0], tofs[db][1]);
            tofs[db][0] += t0;
            tofs[db][1] += t0;
        }
    }
    auto ld_k = [&](int t8, int hb) __attribute__((always_inline)) { return lds_ld_frag(kofs[t8] + hb * 32 * ROW_B); };
    auto ld_v = [&](int t8, int hb) __attribute__((always_inline)) { return lds_ld_frag(kofs[t8] + V_OFF + hb * 32 * ROW_B); };
    auto ld_t = [&](int p, int hb) __attribute__((always_inline)) {
        const int ks = p >> 2, db = p & 3;
        return lds_ld_frag_t(tofs[db][0] + (32 * hb + 16 * ks) * ROW_B, tofs[db][1] + (32 * hb + 16 * ks) * ROW_B);
    };

    u32x4 dsf[2][2];      // dS^T of sub-tile u-1 as B-operand fragments [query block][k-step]
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) dsf[cb][ks] = u32x4{0u, 0u, 0u, 0u};
    bf16x8 ka[8], va[8], ta[8];
    f32x16 x1, y1, x0a, x0b, y0a, y0b;

    // Iteration u (half hb of tile T).  Groups 0-15: dQ^T += K^T dS^T(u-1) on the matrix cores
    // while the vector ALU turns query block 1 of sub-tile u into dS^T; groups 16-47: S^T(u+1),
    // dP^T(u+1) (block 1's overwrite what was just consumed) while the vector ALU does block 0.
    auto stage = [&](auto hb_tag, auto masked_tag, bool pre, int j0, f32x16& x0in, f32x16& y0in, f32x16& x0out,
                     f32x16& y0out, const TileSrc& ts, uint32_t tbump) __attribute__((always_inline)) {
        constexpr int hb = decltype(hb_tag)::value;
        constexpr bool MASKED = decltype(masked_tag)::value;
        if (MASKED) {
            // the last score products of the previous iteration were issued only two groups ago
            // and the compiler does not know they are matrix-core results: let them retire
            asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
            mask1(x0in, 0, pre, j0 + 32 * hb);
            mask1(x1, 1, pre, j0 + 32 * hb);
        }
        pin();
        float w0[16], w1[16], e0[16], e1[16];
        u32x4 dn[2][2];
        static_for<48>([&](auto gc) __attribute__((always_inline)) {
            constexpr int g = decltype(gc)::value;
            if (g < 16) {
                const int ks = g >> 3, db = (g >> 1) & 3, cb = g & 1;
                acc[db][cb] = mma(ta[4 * ks + db], __builtin_bit_cast(bf16x8, dsf[cb][ks]), acc[db][cb]);
            } else {
                const int j = g - 16, t8 = j >> 2, which = j & 3;   // block 1 first: its results are read first
                if (which == 0)      { if (t8 == 0) mma_vd_zero(x1, ka[0], qf[1][0]); else mma_vd(x1, ka[t8], qf[1][t8]); }
                else if (which == 1) { if (t8 == 0) mma_vd_first(y1, va[0], gf[1][0], ndi[1]); else mma_vd(y1, va[t8], gf[1][t8]); }
                else if (which == 2) { if (t8 == 0) mma_vd_zero(x0out, ka[0], qf[0][0]); else mma_vd(x0out, ka[t8], qf[0][t8]); }
                else                 { if (t8 == 0) mma_vd_first(y0out, va[0], gf[0][0], ndi[0]); else mma_vd(y0out, va[t8], gf[0][t8]); }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (hb == 0 && g >= 16 && g < 24) dma_piece(ts, g - 16);
            // transposed K fragments of sub-tile u-1 (groups 0-8) and, for the next iteration, u
            if (g <= 4 && !(g & 1)) ta[5 + (g >> 1)] = ld_t(5 + (g >> 1), 1 - hb);
            if (hb == 0 && g >= 5 && g < 9) {       // then the addresses move on to tile T
                tofs[g - 5][0] += tbump;
                tofs[g - 5][1] += tbump;
            }
            // (in the odd groups 17-25, which carry no other LDS read and no vector ALU work: every LDS
            // read of an iteration is out by group 36, and the wait in front of the tile barrier finds none)
            if (g >= 17 && g <= 25 && (g & 1)) ta[(g - 17) >> 1] = ld_t((g - 17) >> 1, hb);
            // row-wise fragments of sub-tile u+1
            if (g >= 6 && g <= 34 && ((g - 6) & 3) == 0) ka[(g - 6) >> 2] = ld_k((g - 6) >> 2, hb ? 0 : 1);
            if (g >= 8 && g <= 36 && ((g - 8) & 3) == 0) va[(g - 8) >> 2] = ld_v((g - 8) >> 2, hb ? 0 : 1);
            // The LDS reads go out right behind the matrix-core instruction, the vector ALU work
            // follows; its exponential and the product that consumes it sit a group apart (a
            // transcendental's consumer right behind it costs a wait state).
            __builtin_amdgcn_sched_barrier(0);
            // vector ALU: block 1 element g (groups 0-15), block 0 element (g-16)/2 (even groups after)
            if (g < 16) {
                e1[g] = fast_exp2(CART_PRESCALE ? x1[g] + nl2[1] : fmaf(x1[g], c, nl2[1]));
                if (g >= 1) w1[g - 1] = e1[g - 1] * y1[g - 1];
                if (g >= 3 && (g & 1)) dn[1][(g - 3) >> 3][((g - 3) & 7) >> 1] = pack_bf16x2(w1[g - 3], w1[g - 2]);
            } else if (!(g & 1)) {
                const int r = (g - 16) >> 1;
                if (r == 0) w1[15] = e1[15] * y1[15];
                if (r == 1) dn[1][1][3] = pack_bf16x2(w1[14], w1[15]);
                e0[r] = fast_exp2(CART_PRESCALE ? x0in[r] + nl2[0] : fmaf(x0in[r], c, nl2[0]));
                if (r >= 1) w0[r - 1] = e0[r - 1] * y0in[r - 1];
                if (r >= 3 && (r & 1)) dn[0][(r - 3) >> 3][((r - 3) & 7) >> 1] = pack_bf16x2(w0[r - 3], w0[r - 2]);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        w0[15] = e0[15] * y0in[15];
        dn[0][1][3] = pack_bf16x2(w0[14], w0[15]);
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) dsf[cb][ks] = dn[cb][ks];
        __builtin_amdgcn_sched_barrier(0);
    };
    auto settle = [&]() __attribute__((always_inline)) { asm volatile("s_nop 15\n\ts_nop 7" ::: "memory"); };

    {   // prologue: tiles 0 and 1 on their way, scores of sub-tile 0
        const TileSrc t0 = tile_src(0, 0);
#pragma unroll
        for (int n = 0; n < 8; ++n) dma_piece(t0, n);
        dma_wait();
        __syncthreads();
        const TileSrc t1 = tile_src(min(1, nT - 1), 1);
#pragma unroll
        for (int n = 0; n < 8; ++n) dma_piece(t1, n);
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) { ka[t8] = ld_k(t8, 0); va[t8] = ld_v(t8, 0); }
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) {
            if (t8 == 0) { mma_vd_zero(x0a, ka[0], qf[0][0]); mma_vd_zero(x1, ka[0], qf[1][0]);
                           mma_vd_first(y0a, va[0], gf[0][0], ndi[0]); mma_vd_first(y1, va[0], gf[1][0], ndi[1]); }
            else         { mma_vd(x0a, ka[t8], qf[0][t8]); mma_vd(x1, ka[t8], qf[1][t8]);
                           mma_vd(y0a, va[t8], gf[0][t8]); mma_vd(y1, va[t8], gf[1][t8]); }
        }
        settle();
#pragma unroll
        for (int p = 0; p < 5; ++p) ta[p] = ld_t(p, 0);     // placeholder: multiplied by dS = 0
    }
    int buf = 0;
    bool first = true;
    auto tile_iter = [&](int T, auto masked_tag) __attribute__((always_inline)) {
        const int nbuf = buf + 1 == NBUF ? 0 : buf + 1;
        const int nnbuf = nbuf + 1 == NBUF ? 0 : nbuf + 1;
        const TileSrc ts = tile_src(min(T + 2, nT - 1), nnbuf);
        const bool pre = tile_pre(T);
        const int j0 = tile_j0(T);
        const uint32_t fwd = static_cast<uint32_t>(BUF_B), back = static_cast<uint32_t>(-(NBUF - 1) * BUF_B);
        dma_wait();
        __syncthreads();
        // the transposed reads still address tile T-1 when the iteration starts (the very first
        // iteration has no predecessor: its placeholder is tile 0 itself)
        const uint32_t tb = first ? 0u : (buf == 0 ? back : fwd);
        stage(std::integral_constant<int, 0>{}, masked_tag, pre, j0, x0a, y0a, x0b, y0b, ts, tb);
        // the row-wise reads move on to tile T+1 between the two halves
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) kofs[t8] += nbuf == 0 ? back : fwd;
        stage(std::integral_constant<int, 1>{}, masked_tag, pre, j0, x0b, y0b, x0a, y0a, ts, 0u);
        first = false;
        buf = nbuf;
    };
    for (int T = 0; T < nMain; ++T) tile_iter(T, std::false_type{});
    for (int T = nMain; T < nT; ++T) tile_iter(T, std::true_type{});
    {   // drain: dQ^T += K^T dS^T of the last sub-tile (fragments 0-4 are in registers)
        pin();
#pragma unroll
        for (int p = 5; p < 8; ++p) ta[p] = ld_t(p, 1);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                acc[db][0] = mma(ta[4 * ks + db], __builtin_bit_cast(bf16x8, dsf[0][ks]), acc[db][0]);
                acc[db][1] = mma(ta[4 * ks + db], __builtin_bit_cast(bf16x8, dsf[1][ks]), acc[db][1]);
            }
    }
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int qi = wrow0 + 32 * cb + lc;
        f32x16 col[4] = {acc[0][cb], acc[1][cb], acc[2][cb], acc[3][cb]};
        store_rows_bf16(col, qi < S ? dq + ((t0 + qi) * Hq + h) * HD : nullptr, lg, scale);
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

// the fused dK + dV kernel (attn_mfma_bwd_kv.hip)
int bwd_kv_chunk(const cart_attn_desc& d, long tokens, int* n_part);
void launch_attn_bwd_kv(const cart_attn_desc& d, float scale, const bf16_t* Q, const bf16_t* K, const bf16_t* V,
                        const bf16_t* ZK, const bf16_t* ZV, const bf16_t* DO, const float* lse2, const float* delta,
                        bf16_t* dk, bf16_t* dv, float* part_k, float* part_v, const int32_t* cu, int n_tok, int chunk,
                        int n_part, hipStream_t st);

static size_t r256(size_t n) { return (n + 255) & ~static_cast<size_t>(255); }

// beyond the delta array: lse2 (one value per token and head) and the two dZ partial buffers
// [n_part,Hkv,P,128]; packed layout (tokens >= 0 = the packed row count): + the row_lo array.
size_t attn_mfma_bwd_workspace(const cart_attn_desc& d, long tokens) {
    const bool packed = tokens >= 0;
    if (!packed) tokens = static_cast<long>(d.B) * d.S;
    int n_part;
    bwd_kv_chunk(d, tokens, &n_part);
    const size_t rows = r256(static_cast<size_t>(tokens) * d.Hq * sizeof(float));
    const size_t part = r256(static_cast<size_t>(n_part) * d.Hkv * d.P * HD * sizeof(float));
    return rows + 2 * part + (packed ? r256(static_cast<size_t>(tokens) * sizeof(int32_t)) : 0);
}

int launch_attn_bwd_mfma(const cart_attn_desc& d, float scale, const void* q, const void* k,
                         const void* v, const void* zk, const void* zv, const void* o,
                         const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                         float* dzk, float* dzv, void* ws, hipStream_t st, const int32_t* cu, int T) {
    const long tokens = cu ? T : static_cast<long>(d.B) * d.S;
    const size_t rows_b = r256(static_cast<size_t>(tokens) * d.Hq * sizeof(float));
    int n_part;
    const int chunk = bwd_kv_chunk(d, tokens, &n_part);
    const int n_tok = static_cast<int>(tokens);
    const size_t part_b = r256(static_cast<size_t>(n_part) * d.Hkv * d.P * HD * sizeof(float));
    char* w = static_cast<char*>(ws);
    float* delta = reinterpret_cast<float*>(w);
    float* lse2 = reinterpret_cast<float*>(w + rows_b);
    float* part_k = reinterpret_cast<float*>(w + 2 * rows_b);
    float* part_v = reinterpret_cast<float*>(w + 2 * rows_b + part_b);
    // packed batch with a prefix: the dQ kernel cuts its query tiles from the packed rows (it sees
    // one sequence of T rows and the first row of every row's sequence)
    int32_t* row_lo = nullptr;
    if (cu && d.P > 0) {
        row_lo = reinterpret_cast<int32_t*>(w + 2 * rows_b + 2 * part_b);
        launch_row_lo(cu, d.B, T, row_lo, st);
    }
    const bf16_t *Q = static_cast<const bf16_t*>(q), *K = static_cast<const bf16_t*>(k),
                 *V = static_cast<const bf16_t*>(v), *ZK = static_cast<const bf16_t*>(zk),
                 *ZV = static_cast<const bf16_t*>(zv), *DO = static_cast<const bf16_t*>(d_o);
    const float c = scale * CART_LOG2E;
    const bf16_t* O = static_cast<const bf16_t*>(o);
    trace_begin(st);   // kernel order: dq (+ row statistics), dk + dv (one kernel), dz reduce (k, v)
    if (row_lo) {
        const long nQt = (T + BWD_WG_ROWS - 1) / BWD_WG_ROWS;
        hipLaunchKernelGGL(attn_bwd_dq_kernel, dim3(static_cast<unsigned>(nQt * d.Hq)), dim3(256), 0, st, Q, K, V, ZK,
                           ZV, O, DO, lse, lse2, delta, static_cast<bf16_t*>(dq), nullptr, row_lo, n_tok, 1, n_tok,
                           d.Hq, d.Hkv, d.P, c, scale);
    } else {
        const long nQt = (d.S + BWD_WG_ROWS - 1) / BWD_WG_ROWS;
        hipLaunchKernelGGL(attn_bwd_dq_kernel, dim3(static_cast<unsigned>(nQt * d.B * d.Hq)), dim3(256), 0, st, Q, K, V,
                           ZK, ZV, O, DO, lse, lse2, delta, static_cast<bf16_t*>(dq), cu, nullptr, n_tok, d.B, d.S,
                           d.Hq, d.Hkv, d.P, c, scale);
    }
    trace_mark(st);
    launch_attn_bwd_kv(d, scale, Q, K, V, ZK, ZV, DO, lse2, delta, static_cast<bf16_t*>(dk), static_cast<bf16_t*>(dv),
                       part_k, part_v, cu, n_tok, chunk, n_part, st);
    trace_mark(st);
    if (d.P > 0) {
        const long n4 = static_cast<long>(d.Hkv) * d.P * HD / 4;
        const unsigned rg = static_cast<unsigned>((n4 + 255) / 256);
        hipLaunchKernelGGL(dz_reduce_kernel, dim3(rg), dim3(256), 0, st, part_k, dzk, n_part, n4, d.P, d.n_frozen, d.dz_accumulate);
        hipLaunchKernelGGL(dz_reduce_kernel, dim3(rg), dim3(256), 0, st, part_v, dzv, n_part, n4, d.P, d.n_frozen, d.dz_accumulate);
        trace_mark(st);
    }
    return static_cast<int>(hipGetLastError());
}

}  // namespace cart
