// Cartridge attention forward on the matrix cores (bf16 in, fp32 accumulate, head_dim 128):
// Eq. 1 over the cache of Sec. 3.2, [prefix Z (all visible) ; own keys (causal)].
//
// One 256-thread workgroup = 256 consecutive queries of one (sequence, query head); each of its
// four wavefronts owns 64 of them, kept in registers as MFMA operand fragments.  Keys/values
// stream through LDS in tiles of 64 (prefix tiles first, then own tiles up to the diagonal),
// four buffers, one barrier per tile, consumed as sub-tiles of 32 keys.  Per sub-tile a
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
constexpr int FWD_NBUF = 4;     // tile t in buffer t % 4; loads run two tiles ahead of the barrier that publishes them
constexpr int FWD_TILE_B = FWD_BN * ROW_B;

struct FwdSmem {
    char k[FWD_NBUF][FWD_TILE_B];
    char v[FWD_NBUF][FWD_TILE_B];
};

// 1: fold the softmax scale into Q (one extra bf16 rounding of Q) and the softmax reference into
// the score product's init value, so that an exponent costs no arithmetic of its own.  0: scores
// are scaled in fp32, exponent = fma(score, c, -m): exact, one more vector-ALU instruction per
// element.
#ifndef CART_PRESCALE
#define CART_PRESCALE 0
#endif

__global__ __launch_bounds__(256, 1) void attn_fwd_mfma_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ zk, const bf16_t* __restrict__ zv, bf16_t* __restrict__ o,
    float* __restrict__ lse, int* __restrict__ flags, const int32_t* __restrict__ cu,
    const int32_t* __restrict__ row_lo, int n_tok, int B, int Smax, int Hq, int Hkv, int P,
    float c /* scale*log2(e) */) {
    __shared__ FwdSmem sm;
    __shared__ int sm_bad;
    const int G = Hq / Hkv;
    const int nQt = (Smax + FWD_BM - 1) / FWD_BM;
    // workgroup -> (query tile, sequence, head).  KV head is the fastest index so that, with 8
    // KV heads, blockIdx % 8 (the XCD a workgroup lands on) is the KV head and each XCD's L2 keeps
    // one head's prefix; then the query tiles of one sequence, heaviest (longest causal part)
    // first, sequence after sequence: the workgroups running at one time belong to one or two
    // sequences, whose own K/V then stay in L2 (2 % faster than all sequences' heaviest tiles first).
    int id = blockIdx.x;
    const int hk = id % Hkv; id /= Hkv;
    const int g_ = id % G; id /= G;
    const int qt = nQt - 1 - id % nQt;
    const int b = id / nQt;
    const int h = hk * G + g_;
    const int lane = threadIdx.x & 63, lg = lane >> 5, lc = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, in a scalar register
    const int q0 = qt * FWD_BM, wrow0 = q0 + 64 * wv;
    // Rows of sequence b: [t0, t0 + S).  Batched layout: S rows each; packed layout (cu given):
    // rows cu[b] .. cu[b+1]-1 of T, the grid is sized for the longest sequence and a workgroup
    // whose query tile lies past the end of its sequence has nothing to do.
    // Packed layout with a prefix (row_lo given, B = 1, S = all packed rows): query tiles are cut
    // from the packed rows regardless of sequence boundaries -- no sequence ends in a partly
    // filled tile -- and row i sees the own keys row_lo[i] .. i (row_lo = first row of its sequence).
    const SeqSpan sp = seq_span(cu, b, n_tok, Smax, Hq);
    const int S = sp.len;
    const size_t t0 = sp.t0;
    if (q0 >= S) {
        if (threadIdx.x == 0) flags[blockIdx.x] = 0;
        return;
    }
    if (threadIdx.x == 0) sm_bad = 0;

    // this wavefront's 64 queries as B-operand fragments: column = query, k = head element
    // They are pinned to accumulation registers (the matrix cores read B operands from there
    // directly), which leaves the ordinary vector registers to the softmax arithmetic.
    u32x4 qraw[2][8];
    int lo_q[2] = {0, 0};     // first own key the lane's queries see
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        int qi = wrow0 + 32 * cb + lc;
        qi = qi < S ? qi : S - 1;
        if (row_lo) lo_q[cb] = row_lo[qi];
        const bf16_t* qp = q + ((t0 + qi) * Hq + h) * HD + 8 * lg;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const u32x4 w = *reinterpret_cast<const u32x4*>(qp + 16 * t);
#if CART_PRESCALE
            // Q enters every product scaled by c = softmax_scale * log2(e), rounded to bf16 once
            // here: the scores then come out of the matrix cores in log2 units
#pragma unroll
            for (int i = 0; i < 4; ++i)
                qraw[cb][t][i] = pack_bf16x2(__uint_as_float(w[i] << 16) * c, __uint_as_float(w[i] & 0xffff0000u) * c);
#else
            qraw[cb][t] = w;
#endif
        }
    }
    f32x16 acc[4][2];   // O^T: [head-element block][query block]
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][cb][r] = 0.f;
    // keeps Q and the O accumulators in accumulation registers across the loops' control flow
    auto pin = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int t = 0; t < 8; ++t) asm volatile("" : "+a"(qraw[cb][t]));
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) asm volatile("" : "+a"(acc[db][cb]));
    };
    pin();

    // Tile order.  The softmax reference is fixed, so key tiles may come in any order: first every
    // tile all of whose keys are visible to all 256 queries (whole prefix tiles, own tiles below
    // the first query), through a loop without masking code; then the ragged last prefix tile and
    // the (at most four) own tiles on the diagonal, through a copy of the loop that masks.
    const int nPf = P / FWD_BN;                        // whole prefix tiles
    const int rag = (P % FWD_BN) ? 1 : 0;              // ragged prefix tile
    const int own_end = min(S, q0 + FWD_BM);
    // own tiles (of 64 rows from row 0): every query of the workgroup sees the whole of tiles
    // tU0 .. tD-1; tiles tA .. min(tU0, tD)-1 start before the first key of some query and tiles
    // tD .. tEnd-1 lie on the diagonal (one sequence: tA = tU0 = 0)
    const int lo_first = row_lo ? row_lo[q0] : 0, lo_last = row_lo ? row_lo[own_end - 1] : 0;
    const int tA = lo_first / FWD_BN, tU0 = (lo_last + FWD_BN - 1) / FWD_BN, tD = q0 / FWD_BN;
    const int nOf = max(0, tD - tU0);
    const int nLow = min(tU0, tD) - tA;
    const int nMain = nPf + nOf;
    const int nT = nMain + rag + nLow + (own_end + FWD_BN - 1) / FWD_BN - tD;
    const char* zk_b = reinterpret_cast<const char*>(zk) + static_cast<size_t>(hk) * P * ROW_B;
    const char* zv_b = reinterpret_cast<const char*>(zv) + static_cast<size_t>(hk) * P * ROW_B;
    const uint32_t own_pitch = static_cast<uint32_t>(Hkv) * ROW_B;
    const char* k_b = reinterpret_cast<const char*>(k) + (t0 * Hkv + hk) * ROW_B;
    const char* v_b = reinterpret_cast<const char*>(v) + (t0 * Hkv + hk) * ROW_B;
    // tile t of that order: prefix or own, first key (all scalar)
    auto tile_pre = [&](int t) __attribute__((always_inline)) {
        return t < nPf || (rag && t == nMain);
    };
    auto tile_j0 = [&](int t) __attribute__((always_inline)) {
        const int m = t - nMain - rag;      // among the masked own tiles
        return (t < nPf ? t : t < nMain ? tU0 + t - nPf : (rag && t == nMain) ? nPf : m < nLow ? tA + m : tD + m - nLow) * FWD_BN;
    };

    // Direct-to-LDS load of one tile, eight instructions per wavefront (K rows, then V rows),
    // handed out one per matrix-core instruction by the stage below.
    const uint32_t dma_c0 = (lane & 15) ^ (((lane >> 4) & 3) << 2);   // chunk under the swizzle, before ^ i
    struct TileSrc { const char* kb; const char* vb; int lim; uint32_t pitch; uint32_t lds_k, lds_v; };
    auto tile_src = [&](int t, int buf) __attribute__((always_inline)) {
        const bool pre = tile_pre(t);
        const int j0 = tile_j0(t);
        TileSrc ts;
        ts.pitch = pre ? static_cast<uint32_t>(ROW_B) : own_pitch;
        ts.kb = (pre ? zk_b : k_b) + static_cast<size_t>(j0) * ts.pitch;
        ts.vb = (pre ? zv_b : v_b) + static_cast<size_t>(j0) * ts.pitch;
        ts.lim = (pre ? P : S) - 1 - j0;    // rows past the end repeat the last valid row
        ts.lds_k = lds_addr(sm.k[buf]);
        ts.lds_v = lds_addr(sm.v[buf]);
        return ts;
    };
    auto dma_piece = [&](const TileSrc& ts, int n) __attribute__((always_inline)) {
        const int i = n & 3;
        const int r0 = (4 * wv + i) * 4;
        const uint32_t voff = __umul24(min(r0 + (lane >> 4), ts.lim), ts.pitch) + ((dma_c0 ^ i) << 4);
        if (n < 4) dma16(ts.kb, voff, ts.lds_k + r0 * ROW_B);
        else       dma16(ts.vb, voff, ts.lds_v + r0 * ROW_B);
    };
    // hidden entries of the scores of the sub-tile whose first key is j0 (prefix or own) -> very negative
    auto mask = [&](f32x16 (&x)[2], bool pre, int j0) __attribute__((always_inline)) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            // key j0 + d_row(r, lg) is hidden when it exceeds the lane's last visible key
            mask_above(x[cb], (pre ? P - 1 : wrow0 + 32 * cb + lc) - j0 - 4 * lg);
            // ... or precedes the first key of the query's sequence
            if (row_lo && !pre) mask_below(x[cb], lo_q[cb] - j0 - 4 * lg);
        }
    };

    // Per-lane LDS addresses of the operand fragments, complete except for compile-time offsets;
    // they move from buffer to buffer once per tile (K fragments are fetched one tile ahead of V).
    uint32_t kofs[8], vofs[4][2];
    {
        const uint32_t lk = lds_addr(sm.k[1]), lv = lds_addr(sm.v[0]);
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) kofs[t8] = lk + lc * ROW_B + (((2 * t8 + lg) ^ swz(lc)) << 4);
        const int s16 = lane & 15;
        const int row = 4 * lg + (s16 >> 2);
        const int col0 = 16 * ((lane >> 4) & 1) + 4 * (s16 & 3);
        const int half = ((col0 >> 2) & 1) * 8;
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const int ch = (32 * db + col0) >> 3;
            vofs[db][0] = lv + row * ROW_B + ((ch ^ swz(row)) << 4) + half;
            vofs[db][1] = lv + (row + 8) * ROW_B + ((ch ^ swz(row + 8)) << 4) + half;
        }
    }
    typedef const bf16x8 __attribute__((address_space(3))) * lds_b128;
    typedef s16x4 __attribute__((address_space(3))) * lds_b64;
    // row-wise K fragment t8 of the 32-row half hb of the buffer kofs points at
    auto ld_k = [&](int t8, int hb) __attribute__((always_inline)) {
        return *(lds_b128)(kofs[t8] + hb * 32 * ROW_B);
    };
    // transposed V fragment (k-step ks, head-element block db) of half hb of the buffer at vofs
    auto ld_v = [&](int ks, int db, int hb) __attribute__((always_inline)) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_b64)(vofs[db][0] + (32 * hb + 16 * ks) * ROW_B));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_b64)(vofs[db][1] + (32 * hb + 16 * ks) * ROW_B));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };

    // -m (the softmax reference of the lane's query) in all 16 registers of a set: the first
    // product of every score chain starts from it, so S arrives as the exponent c s - m
#if CART_PRESCALE
    f32x16 ninit[2];
#else
    float negm[2];
#endif
    float l_run[2] = {0.f, 0.f};
    // Scores live in ordinary vector registers, in two sets used alternately: while the vector
    // ALU reads S(u) from one set the matrix cores write S(u+1) into the other, so no copy sits
    // between the matrix cores' results and the softmax arithmetic.
    f32x16 sa[2], sb[2];
    u32x4 pf[2][2];           // P^T(u-1) as B-operand fragments [query block][k-step]
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) pf[cb][ks] = u32x4{0u, 0u, 0u, 0u};
    bf16x8 ka[8], va[2][4];   // K fragments of sub-tile u+1, V fragments of sub-tile u-1
    // The last two V fragments have a spare register set each (indexed by the parity of the
    // iteration that USES them): the next iteration's copies are requested before this
    // iteration's last use, so no LDS read is issued in the last groups and the wait in front of
    // the tile barrier finds nothing outstanding.
    bf16x8 vb6[2], vb7[2];

    // Iteration u (sub-tile hb of a tile; MASKED: it may hold hidden keys).  On entry: x = S(u),
    // ka = K fragments of sub-tile u+1, va = V fragments of sub-tile u-1, pf = P(u-1); on exit
    // y = S(u+1).  The work is laid out as 32 groups of one matrix-core instruction plus one
    // softmax element and the odd jobs that go with it, fenced so that the scheduler keeps the
    // spread: the matrix cores run S^T(u+1) = K Q^T (groups 0-15) and O^T += V^T P^T(u-1)
    // (groups 16-31) while the vector ALU turns S(u) into P(u); each fragment register is
    // refilled from LDS for the next iteration right after its last use, and the eight
    // direct-to-LDS loads of tile t+2 (DMA, first sub-tile only) ride along in groups 0-7.
    auto stage = [&](auto hb_tag, auto masked_tag, bool pre, int j0, f32x16 (&x)[2], f32x16 (&y)[2],
                     const TileSrc& ts) __attribute__((always_inline)) {
        constexpr int hb = decltype(hb_tag)::value;
        constexpr bool MASKED = decltype(masked_tag)::value;
        if (MASKED) mask(x, pre, j0 + 32 * hb);
        pin();
        float pe[32];
        u32x4 pn[2][2];
#pragma unroll
        for (int g = 0; g < 32; ++g) {
            if (g < 16) {
                const int t8 = g >> 1, cb = g & 1;
#if CART_PRESCALE
                if (t8 == 0) mma_vd_first(y[cb], ka[0], qraw[cb][0], ninit[cb]);
#else
                if (t8 == 0) mma_vd_zero(y[cb], ka[0], qraw[cb][0]);
#endif
                else         mma_vd(y[cb], ka[t8], qraw[cb][t8]);
            } else {
                const int i = g - 16, ks = i >> 3, db = (i >> 1) & 3, cb = i & 1, p = 4 * ks + db;
                const bf16x8 vf_ = p == 6 ? vb6[hb] : p == 7 ? vb7[hb] : va[ks][db];
                acc[db][cb] = mma(vf_, __builtin_bit_cast(bf16x8, pf[cb][ks]), acc[db][cb]);
            }
            __builtin_amdgcn_sched_barrier(0);   // the matrix-core instruction leads its group
            if (hb == 0 && g < 8) dma_piece(ts, g);
            // refill the fragment register the previous two groups used last
            if (g >= 2 && g <= 16 && !(g & 1)) ka[(g - 2) >> 1] = ld_k((g - 2) >> 1, hb);
            if (g >= 18 && g <= 28 && !(g & 1)) {
                const int i = g - 18;
                va[i >> 3][(i >> 1) & 3] = ld_v(i >> 3, (i >> 1) & 3, hb);
            }
            if (g == 25) vb6[1 - hb] = ld_v(1, 2, hb);
            if (g == 27) vb7[1 - hb] = ld_v(1, 3, hb);
            // the LDS reads go out right behind the matrix-core instruction, ahead of the vector ALU work
            __builtin_amdgcn_sched_barrier(0);
            {   // softmax element g; the pair before it is rounded, packed and summed
                const int cb = g >> 4, r = g & 15;
#if CART_PRESCALE
                pe[g] = fast_exp2(x[cb][r]);
#else
                pe[g] = fast_exp2(fmaf(x[cb][r], c, negm[cb]));
#endif
                if (g >= 2 && !(g & 1)) {
                    const int e = g - 2, cbe = e >> 4, re = e & 15;
                    pn[cbe][re >> 3][(re & 7) >> 1] = pack_bf16x2(pe[e], pe[e + 1]);
                    l_run[cbe] += pe[e] + pe[e + 1];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        pn[1][1][3] = pack_bf16x2(pe[30], pe[31]);
        l_run[1] += pe[30] + pe[31];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) pf[cb][ks] = pn[cb][ks];
        __builtin_amdgcn_sched_barrier(0);
    };
    // the matrix-core results of the inline-assembly products are not tracked by the compiler's
    // hazard logic: before the vector ALU touches them, let the last one retire
    auto settle = [&]() __attribute__((always_inline)) { asm volatile("s_nop 15\n\ts_nop 7" ::: "memory"); };

    {   // tiles 0 and 1 on their way; scores of sub-tile 0 and the softmax reference of every
        // query: its maximum over that sub-tile (which holds a visible key for every query)
        const TileSrc t0 = tile_src(0, 0);
#pragma unroll
        for (int n = 0; n < 8; ++n) dma_piece(t0, n);
        const TileSrc t1 = tile_src(min(1, nT - 1), 1);
#pragma unroll
        for (int n = 0; n < 8; ++n) dma_piece(t1, n);
        const TileSrc t2 = tile_src(min(2, nT - 1), 2);
#pragma unroll
        for (int n = 0; n < 8; ++n) dma_piece(t2, n);
        dma_wait_but<16>();
        __syncthreads();
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) ka[t8] = lds_frag_n(sm.k[0], lc, 16 * t8 + 8 * lg);
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) {
            if (t8 == 0) { mma_vd_zero(sa[0], ka[0], qraw[0][0]); mma_vd_zero(sa[1], ka[0], qraw[1][0]); }
            else         { mma_vd(sa[0], ka[t8], qraw[0][t8]);    mma_vd(sa[1], ka[t8], qraw[1][t8]); }
        }
        settle();
        mask(sa, tile_pre(0), tile_j0(0));
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            float tm = sa[cb][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) tm = fmaxf(tm, sa[cb][r]);
#if CART_PRESCALE
            const float nm = -partner_max(tm);
#pragma unroll
            for (int r = 0; r < 16; ++r) { ninit[cb][r] = nm; sa[cb][r] += nm; }
#else
            negm[cb] = -partner_max(tm) * c;
#endif
        }
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) ka[t8] = lds_frag_n(sm.k[0], 32 + lc, 16 * t8 + 8 * lg);   // sub-tile 1
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)     // placeholder for "V of sub-tile -1": multiplied by P = 0
#pragma unroll
            for (int db = 0; db < 4; ++db) va[ks][db] = lds_frag_t(sm.v[0], 16 * ks, 32 * db, lane);
        vb6[0] = va[1][2];
        vb7[0] = va[1][3];
    }
    // Four LDS buffers, tile t in buffer t % 4.  The one barrier per tile opens the iteration of
    // the tile's first sub-tile: it publishes tile t+1 (read from this iteration on; its loads
    // went out two iterations ago, so their memory latency is covered twice over) and retires
    // tile t-1's buffer (its last fragments were fetched in the previous iteration), which then
    // receives tile t+3.
    int buf = 0;
    auto tile_iter = [&](int t, auto masked_tag) __attribute__((always_inline)) {
        const int nbuf = buf + 1 == FWD_NBUF ? 0 : buf + 1;
        const int nnbuf = nbuf + 1 == FWD_NBUF ? 0 : nbuf + 1;
        const int n3buf = nnbuf + 1 == FWD_NBUF ? 0 : nnbuf + 1;
        const TileSrc ts = tile_src(min(t + 3, nT - 1), n3buf);
        const bool pre = tile_pre(t);
        const int j0 = tile_j0(t);
        dma_wait_but<8>();      // tile t+1 has landed (t+2 may still be in flight)
        __syncthreads();
        if (decltype(masked_tag)::value && !pre && j0 > wrow0 + 63) {
            // A diagonal tile that lies entirely behind this wavefront's 64 queries (so do all
            // that follow): nothing to compute -- its share of the loads still goes out, and the
            // state of the pipeline (P and the V fragments of the last visible sub-tile) waits
            // for the drain.  The products skipped are a few per cent of the kernel's, and under
            // these kernels the chip's clock follows the energy spent.
#pragma unroll
            for (int n = 0; n < 8; ++n) dma_piece(ts, n);
        } else {
            stage(std::integral_constant<int, 0>{}, masked_tag, pre, j0, sa, sb, ts);
            stage(std::integral_constant<int, 1>{}, masked_tag, pre, j0, sb, sa, ts);
        }
        // fragment addresses follow the buffers: K to tile t+2's, V to tile t+1's
        const uint32_t dk = nnbuf == 0 ? static_cast<uint32_t>(-(FWD_NBUF - 1) * FWD_TILE_B) : static_cast<uint32_t>(FWD_TILE_B);
        const uint32_t dv = nbuf == 0 ? static_cast<uint32_t>(-(FWD_NBUF - 1) * FWD_TILE_B) : static_cast<uint32_t>(FWD_TILE_B);
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) kofs[t8] += dk;
#pragma unroll
        for (int db = 0; db < 4; ++db) { vofs[db][0] += dv; vofs[db][1] += dv; }
        buf = nbuf;
    };
    for (int t = 0; t < nMain; ++t) tile_iter(t, std::false_type{});
    for (int t = nMain; t < nT; ++t) tile_iter(t, std::true_type{});
    {   // drain: O^T += V^T P^T of the last sub-tile (its V fragments are already in registers)
        pin();
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const int p = 4 * ks + db;
                const bf16x8 vf_ = p == 6 ? vb6[0] : p == 7 ? vb7[0] : va[ks][db];
                acc[db][0] = mma(vf_, __builtin_bit_cast(bf16x8, pf[0][ks]), acc[db][0]);
                acc[db][1] = mma(vf_, __builtin_bit_cast(bf16x8, pf[1][ks]), acc[db][1]);
            }
    }
#if CART_PRESCALE
    float m_ref[2] = {-ninit[0][0], -ninit[1][0]};
#else
    float m_ref[2] = {-negm[0], -negm[1]};
#endif

    // normalise and store: lane holds, for its query, head elements 32db + 8(r/4) + 4g + r%4
    bool bad = false;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int qi = wrow0 + 32 * cb + lc;
        const float l_tot = l_run[cb] + partner(l_run[cb]);
        const float inv = 1.f / l_tot;
        float chk = 0.f;
        if (qi < S) {
            bf16_t* op = o + ((t0 + qi) * Hq + h) * HD;
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
                lse[sp.stat_b + h * sp.stat_h + qi] = (m_ref[cb] + fast_log2(l_tot)) * CART_LN2;
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
    float* __restrict__ lse, const int* __restrict__ flags, const int32_t* __restrict__ cu,
    const int32_t* __restrict__ row_lo, int n_tok, int B, int Smax, int Hq, int Hkv, int P, float c) {
    if (flags[blockIdx.x] == 0) return;
    const int G = Hq / Hkv;
    const int nQt = (Smax + FWD_BM - 1) / FWD_BM;
    int id = blockIdx.x;
    const int hk = id % Hkv; id /= Hkv;
    const int g_ = id % G; id /= G;
    const int qt = nQt - 1 - id % nQt;
    const int b = id / nQt;
    const int h = hk * G + g_;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const SeqSpan sp = seq_span(cu, b, n_tok, Smax, Hq);
    const int S = sp.len;
    const size_t t0 = sp.t0;
    for (int i = qt * FWD_BM + wv; i < min(S, (qt + 1) * FWD_BM); i += 4) {
        const size_t row = (t0 + i) * Hq + h;
        const uint32_t qw = *reinterpret_cast<const uint32_t*>(q + row * HD + 2 * lane);
        const float q0 = __uint_as_float(qw << 16), q1 = __uint_as_float(qw & 0xffff0000u);
        float m = -3.0e38f, l = 0.f, a0 = 0.f, a1 = 0.f;
        const int own0 = row_lo ? row_lo[i] : 0;      // first own key of the row
        for (int j = 0; j < P + (i - own0) + 1; ++j) {
            const size_t kr = j < P ? static_cast<size_t>(hk) * P + j
                                    : (t0 + own0 + (j - P)) * Hkv + hk;
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
        if (lane == 0) lse[sp.stat_b + h * sp.stat_h + i] = (m + fast_log2(l)) * CART_LN2;
    }
}

// row_lo[i] = first packed row of the sequence that row i belongs to (cu: B+1 offsets, cu[B] = T)
__global__ __launch_bounds__(256) void attn_row_lo_kernel(const int32_t* __restrict__ cu, int B, int T,
                                                          int32_t* __restrict__ row_lo) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= T) return;
    int lo = 0, hi = B;                 // largest b with cu[b] <= i
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] <= i) lo = mid; else hi = mid;
    }
    row_lo[i] = cu[lo];
}
int launch_row_lo(const int32_t* cu, int B, int T, int32_t* row_lo, hipStream_t st) {
    hipLaunchKernelGGL(attn_row_lo_kernel, dim3((T + 255) / 256), dim3(256), 0, st, cu, B, T, row_lo);
    return static_cast<int>(hipGetLastError());
}

bool attn_mfma_supported(const cart_attn_desc& d) {
    return d.dtype == CART_BF16 && d.D == 128;
}
// workgroups: per sequence, or over the packed rows (a packed batch with a prefix; T > 0)
static long fwd_grid(const cart_attn_desc& d, int T) {
    if (T > 0 && d.P > 0) return static_cast<long>((T + FWD_BM - 1) / FWD_BM) * d.Hq;
    return static_cast<long>((d.S + FWD_BM - 1) / FWD_BM) * d.B * d.Hq;
}
static size_t r256(size_t n) { return (n + 255) & ~static_cast<size_t>(255); }
// one overflow flag per workgroup; packed batches: + the first row of every row's sequence
size_t attn_mfma_fwd_workspace(const cart_attn_desc& d, int T) {
    return r256(static_cast<size_t>(fwd_grid(d, T)) * sizeof(int)) + (T > 0 ? r256(static_cast<size_t>(T) * sizeof(int32_t)) : 0);
}

// cu == nullptr: batched layout [B,S,...].  Otherwise the packed layout: d.S is the longest
// sequence, T the number of packed rows, cu (device) the B+1 row offsets.
int launch_attn_fwd_mfma(const cart_attn_desc& d, float scale, const void* q, const void* k,
                         const void* v, const void* zk, const void* zv, void* o, float* lse,
                         void* ws, hipStream_t st, const int32_t* cu, int T) {
    if (!cu) T = 0;
    const unsigned grid = static_cast<unsigned>(fwd_grid(d, T));
    int* flags = static_cast<int*>(ws);
    int32_t* row_lo = nullptr;
    int B = d.B, S = d.S;
    const bf16_t *Q = static_cast<const bf16_t*>(q), *K = static_cast<const bf16_t*>(k),
                 *V = static_cast<const bf16_t*>(v), *ZK = static_cast<const bf16_t*>(zk),
                 *ZV = static_cast<const bf16_t*>(zv);
    if (cu && d.P > 0) {   // tiles over the packed rows: the kernels see one sequence of T rows
        row_lo = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + r256(static_cast<size_t>(grid) * sizeof(int)));
        launch_row_lo(cu, d.B, T, row_lo, st);
        cu = nullptr;
        B = 1;
        S = T;
    }
    trace_begin(st);   // kernel order: forward, repair
    hipLaunchKernelGGL(attn_fwd_mfma_kernel, dim3(grid), dim3(256), 0, st, Q, K, V, ZK, ZV,
                       static_cast<bf16_t*>(o), lse, flags, cu, row_lo, T, B, S, d.Hq, d.Hkv, d.P, scale * CART_LOG2E);
    trace_mark(st);
    hipLaunchKernelGGL(attn_fwd_repair_kernel, dim3(grid), dim3(256), 0, st, Q, K, V, ZK, ZV,
                       static_cast<bf16_t*>(o), lse, flags, cu, row_lo, T, B, S, d.Hq, d.Hkv, d.P, scale * CART_LOG2E);
    trace_mark(st);
    return static_cast<int>(hipGetLastError());
}

}  // namespace cart
