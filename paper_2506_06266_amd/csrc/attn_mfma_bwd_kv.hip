// Key and value gradients of cartridge attention in ONE pass over the queries (bf16, head_dim
// 128): dK, dV of the own tokens and the per-chunk partials of dZ_k, dZ_v (Sec. 3.2: the loss is
// back-propagated into the key and value vectors of Z with the model frozen).
//
// Keys stationary, as in the split dK / dV kernels this replaces, but the scores S and the
// probabilities P are formed once and serve both gradients: 4 contractions per visible (query,
// key) pair (S, dP, dV, dK) instead of 5 (S twice).  One wavefront cannot hold the accumulators of
// both gradients for 64 keys next to the stationary K and V fragments (that is 384 of its 512
// registers before any working set), so the work of a block of 64 keys is split over a PAIR of
// wavefronts on two SIMDs that stream the same Q / dO tiles from LDS:
//   wavefront A ("P"):   S = Q K^T,  P = 2^(c S - lse2),            dV^T += dO^T P
//   wavefront B ("dS"):  dP = dO V^T - delta,  dS = P (dP - delta),  dK^T += Q^T dS
// A hands P over as the bf16 operand fragments it feeds to its own dV product, through a
// double-buffered 4 KB LDS slot; B runs one sub-tile (32 query rows) behind A, so a slot is
// written in one iteration and read in the next, with the workgroup's barrier between them.  A
// workgroup is two such pairs = 128 keys of one (sequence | chunk of token rows, KV head).
//
// Everything else follows the other backward kernels: Q / dO tiles of 64 rows go straight to LDS
// (direct loads, four buffers), each iteration is 32 fenced groups of one matrix-core instruction
// plus its share of LDS reads and vector-ALU work, tiles that need no mask run through a loop
// without masking code, and prefix-slot gradients leave as fp32 partials per chunk of token rows.
#include "attn_mfma.h"

namespace cart {
using namespace mfma;

constexpr int KV_TILE = 64;                       // token rows per LDS tile (two sub-tiles of 32)
constexpr int KV_TILE_B = KV_TILE * ROW_B;
constexpr int KV_NBUF = 4;
constexpr int KV_BUF_B = 2 * KV_TILE_B;           // one buffer: Q tile, dO tile
constexpr int KV_G_OFF = KV_TILE_B;               // dO tile inside a buffer
constexpr int KV_WG_KEYS = 128;                   // keys per workgroup: two pairs of wavefronts x 64
constexpr int KV_SLOT_B = 4096;                   // P of one sub-tile for 64 keys: 4 fragments x 64 lanes x 16 B
#ifndef KV_PREFIX_WGS
#define KV_PREFIX_WGS 512                         // prefix workgroups aimed at when the token rows are cut into chunks
#endif
constexpr int KV_MIN_CHUNK = 2048;

struct KvSmem {
    struct { char q[KV_TILE_B]; char g[KV_TILE_B]; } t[KV_NBUF];
    float nl2[KV_NBUF][KV_TILE];
    float ndl[KV_NBUF][KV_TILE];
    char slot[2][2][KV_SLOT_B];                   // [pair][sub-tile parity]
};

// One LDS block for the workgroup, at file scope: the two roles are separate (not inlined)
// functions, each with a register allocation of its own, that address the same memory.
__shared__ KvSmem kv_sm;

// The workgroup barrier without the wait for every outstanding LDS and memory operation that
// __syncthreads() puts in front of it: in the hot loop a wavefront only has to have finished what
// the OTHER wavefronts are about to depend on (A: its direct-to-LDS loads and its P-slot writes;
// B: nothing), and fragment loads for later iterations stay in flight across the barrier.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }
__device__ __forceinline__ void lds_wait0() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

__device__ __forceinline__ void kv_store_f32(const f32x16 (&acc)[4], float* row_ptr, int lg, float mul) {
    if (!row_ptr) return;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            f32x4 w = {acc[db][4 * r4] * mul, acc[db][4 * r4 + 1] * mul, acc[db][4 * r4 + 2] * mul, acc[db][4 * r4 + 3] * mul};
            *reinterpret_cast<f32x4*>(row_ptr + 32 * db + 8 * r4 + 4 * lg) = w;
        }
}
__device__ __forceinline__ void kv_store_bf16(const f32x16 (&acc)[4], bf16_t* row_ptr, int lg, float mul) {
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

// The kernel's arguments.  The role functions are real calls, and a call passes its arguments in
// vector registers; they get one pointer -- the kernel-argument segment, taken in the kernel itself
// (the builtin that returns it is only meaningful there: inside a called function it yields a null
// pointer) -- make it wave-uniform again and read this block through the scalar cache, so that
// every pointer and size stays in scalar registers.
struct KvArgs {
    const bf16_t *q, *k, *v, *zk, *zv, *d_o;
    const float *nlse2, *ndelta;
    bf16_t *dk_own, *dv_own;
    float *part_k, *part_v;
    const int32_t* cu;
    int n_tok, chunk, B, Smax, Hq, Hkv, P;
    float c, scale;
};

template <bool roleB>
__device__ __attribute__((noinline)) void kv_role(const KvArgs* args_generic) {
    const uint64_t au = reinterpret_cast<uint64_t>(args_generic);
    const uint32_t a_hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(au >> 32)));
    const uint32_t a_lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<uint32_t>(au)));
    const uint64_t as = (static_cast<uint64_t>(a_hi) << 32) | static_cast<uint64_t>(a_lo);
#if defined(__HIP_DEVICE_COMPILE__)
    const KvArgs a = *(const __attribute__((address_space(4))) KvArgs*)as;
#else
    const KvArgs a = *reinterpret_cast<const KvArgs*>(as);      // (host pass: never runs)
#endif
    const bf16_t* __restrict__ q = a.q; const bf16_t* __restrict__ k = a.k; const bf16_t* __restrict__ v = a.v;
    const bf16_t* __restrict__ zk = a.zk; const bf16_t* __restrict__ zv = a.zv; const bf16_t* __restrict__ d_o = a.d_o;
    const float* __restrict__ nlse2 = a.nlse2; const float* __restrict__ ndelta = a.ndelta;
    bf16_t* __restrict__ dk_own = a.dk_own; bf16_t* __restrict__ dv_own = a.dv_own;
    float* __restrict__ part_k = a.part_k; float* __restrict__ part_v = a.part_v;
    const int32_t* __restrict__ cu = a.cu;
    const int n_tok = a.n_tok, chunk = a.chunk, Smax = a.Smax, Hq = a.Hq, Hkv = a.Hkv, P = a.P;
    const float c = a.c, scale = a.scale;
    KvSmem& sm = kv_sm;
    const int G = Hq / Hkv;
    const int nPb = (P + KV_WG_KEYS - 1) / KV_WG_KEYS, nOb = (Smax + KV_WG_KEYS - 1) / KV_WG_KEYS;
    // workgroup -> (KV head, key block, chunk of token rows | sequence): KV head fastest; the
    // prefix blocks (long streams: every token row of a chunk, all G heads) first
    int id = blockIdx.x;
    const int hk = id % Hkv; id /= Hkv;
    int kb_, b_;
    SeqSpan sp;
    const int nChunk = (n_tok + chunk - 1) / chunk;
    if (id < nPb * nChunk) {
        kb_ = id % nPb;
        b_ = id / nPb;
        sp.t0 = static_cast<size_t>(b_) * chunk;
        sp.len = min(chunk, n_tok - b_ * chunk);
        sp.stat_b = sp.stat_h = 0;
    } else {
        id -= nPb * nChunk;
        kb_ = nPb + id % nOb;
        b_ = id / nOb;
        sp = seq_span(cu, b_, n_tok, Smax, Hq);
    }
    const int kb = kb_, b = b_;      // for a prefix block b is the chunk
    const bool pre = kb < nPb;
    const int key0 = (pre ? kb : kb - nPb) * KV_WG_KEYS;
    const int S = sp.len;
    const size_t t0 = sp.t0;
    const int nkeys = pre ? P : S;
    const int lane = threadIdx.x & 63, lg = lane >> 5, lc = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int pair = wv >> 1;
    const int wkey0 = key0 + 64 * pair;
    if (!pre && key0 >= S) return;

    // this wavefront's 64 keys as B operands (column = key, k = head element): K for A, V for B
    u32x4 sf[2][8];
#pragma unroll
    for (int kc = 0; kc < 2; ++kc) {
        const int key = min(wkey0 + 32 * kc + lc, nkeys - 1);
        const size_t row = pre ? static_cast<size_t>(hk) * P + key : (t0 + key) * Hkv + hk;
        const bf16_t* sp_ = (roleB ? (pre ? zv : v) : (pre ? zk : k)) + row * HD + 8 * lg;
#pragma unroll
        for (int t = 0; t < 8; ++t) sf[kc][t] = *reinterpret_cast<const u32x4*>(sp_ + 16 * t);
    }
    f32x16 acc[4][2];   // dV^T (A) or dK^T (B): [head-element block][key block]
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][kc][r] = 0.f;
    auto pin = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
            for (int t = 0; t < 8; ++t) asm volatile("" : "+a"(sf[kc][t]));
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int kc = 0; kc < 2; ++kc) asm volatile("" : "+a"(acc[db][kc]));
    };
    pin();

    // The stream of query tiles (64 token rows of one head): per head the whole tiles entirely
    // after the block's last key need no mask, the tiles on the diagonal and the ragged last tile
    // do.  Order: the unmasked tiles of every head, then the masked tiles of every head.
    const int nQtAll = (S + KV_TILE - 1) / KV_TILE, nFullEnd = S / KV_TILE;
    const int qt0 = pre ? 0 : key0 / KV_TILE;
    const int qtF0 = pre ? 0 : qt0 + KV_WG_KEYS / KV_TILE;
    const int nFull = max(0, nFullEnd - qtF0);
    const int nM1 = min(qtF0, nQtAll) - qt0;
    const int nM = nM1 + ((nFullEnd < nQtAll && nFullEnd >= qtF0) ? 1 : 0);
    const int nMain = G * nFull, nT = G * (nFull + nM);
    const char* q_c = reinterpret_cast<const char*>(q);
    const char* g_c = reinterpret_cast<const char*>(d_o);
    const uint32_t q_pitch = static_cast<uint32_t>(Hq) * ROW_B;
    int it_ph = nFull > 0 ? 0 : 1, it_g = 0, it_n = 0, it_cnt = 0;
    struct TileSrc { const char* qb; const char* gb; const char* rb; int lim; int i0; uint32_t lds_q, lds_g, lds_r; };
    const uint32_t dma_c0 = (lane & 15) ^ (((lane >> 4) & 3) << 2);
    auto next_tile = [&](int buf) __attribute__((always_inline)) {
        const int qt = it_ph == 0 ? qtF0 + it_n : (it_n < nM1 ? qt0 + it_n : nFullEnd);
        const int h = hk * G + it_g;
        TileSrc ts;
        ts.i0 = qt * KV_TILE;
        const size_t base = (t0 * Hq + h) * ROW_B + static_cast<size_t>(ts.i0) * q_pitch;
        ts.qb = q_c + base;
        ts.gb = g_c + base;
        ts.lim = S - 1 - ts.i0;
        ts.rb = reinterpret_cast<const char*>((pair ? ndelta : nlse2) + static_cast<size_t>(h) * n_tok + t0 + ts.i0);
        ts.lds_q = lds_addr(sm.t[buf].q);
        ts.lds_g = lds_addr(sm.t[buf].g);
        ts.lds_r = lds_addr(pair ? sm.ndl[buf] : sm.nl2[buf]);
        if (it_cnt < nT - 1) {     // past the end the last tile is fetched again, into a retired buffer
            ++it_cnt;
            ++it_n;
            if (it_n == (it_ph == 0 ? nFull : nM)) {
                it_n = 0;
                if (++it_g == G) { it_g = 0; ++it_ph; }
            }
        }
        return ts;
    };
    // Direct-to-LDS loads of a tile, all issued by the two A wavefronts (B is the busier role):
    // seventeen each -- 8 x 4 Q rows, 8 x 4 dO rows of the wavefront's half of the tile, and one
    // of the two row-value arrays (pair 0: -lse2, pair 1: -delta).
    auto dma_piece = [&](const TileSrc& ts, int n) __attribute__((always_inline)) {
        if (n == 16) {
            dma4(ts.rb, static_cast<uint32_t>(min(lane, ts.lim)) * 4u, ts.lds_r);
            return;
        }
        const int i = n & 7;
        const int r0 = (8 * pair + i) * 4;
        const uint32_t voff = __umul24(min(r0 + (lane >> 4), ts.lim), q_pitch) + ((dma_c0 ^ (i & 3)) << 4);
        if (n < 8) dma16(ts.qb, voff, ts.lds_q + r0 * ROW_B);
        else       dma16(ts.gb, voff, ts.lds_g + r0 * ROW_B);
    };
    constexpr int KV_DMA = 17, KV_DMA0 = 9;      // pieces per tile; how many of them ride in the first half

    const uint32_t fwd = static_cast<uint32_t>(KV_BUF_B), back = static_cast<uint32_t>(-(KV_NBUF - 1) * KV_BUF_B);
    const uint32_t rfwd = static_cast<uint32_t>(KV_TILE * 4), rback = static_cast<uint32_t>(-(KV_NBUF - 1) * KV_TILE * 4);
    const uint32_t slot0 = lds_addr(sm.slot[pair][0]) + lane * 16;     // fragment f of parity s: + s * SLOT_B + f * 1024

    if constexpr (!roleB) {
        // =========================================================================================
        // A: S, P, dV.  Iteration u (half hb of tile T): on entry xin = S(u), qa = row-wise Q
        // fragments of sub-tile u+1, nl = -lse2 of sub-tile u, ta = transposed dO fragments of
        // sub-tile u-1, xf = P(u-1).  Matrix cores: S(u+1) (groups 0-15), dV^T += dO^T P(u-1)
        // (groups 16-31); vector ALU: P(u), which goes to the pair's slot at the end.
        // =========================================================================================
        uint32_t qofs[8], tofs[4][2], rofs, rofs_c;
        {
            const uint32_t t1 = lds_addr(sm.t[1].q), tg0 = lds_addr(sm.t[0].g);
#pragma unroll
            for (int t8 = 0; t8 < 8; ++t8) qofs[t8] = t1 + frag_n_ofs(lane, t8);
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                frag_t_ofs(lane, db, tofs[db][0], tofs[db][1]);
                tofs[db][0] += tg0;
                tofs[db][1] += tg0;
            }
            rofs = lds_addr(&sm.nl2[1][4 * lg]);
            rofs_c = lds_addr(&sm.nl2[0][4 * lg]);
        }
        auto ld_q = [&](int t8, int hb) __attribute__((always_inline)) { return lds_ld_frag(qofs[t8] + hb * 32 * ROW_B); };
        auto ld_t = [&](int p, int hb) __attribute__((always_inline)) {
            const int ks = p >> 2, db = p & 3;
            return lds_ld_frag_t(tofs[db][0] + (32 * hb + 16 * ks) * ROW_B, tofs[db][1] + (32 * hb + 16 * ks) * ROW_B);
        };
        auto ld_rows_at = [&](f32x16& d, uint32_t base, int hb) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const f32x4 w = lds_ld_f32x4(base + (32 * hb + 8 * j) * 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) d[4 * j + e] = w[e];
            }
        };
        // a query row of the sub-tile starting at token i0 is hidden from a key when it precedes
        // it (own keys) or lies past the end of the sequence (clamped tile rows)
        auto mask1 = [&](f32x16& x, int kc, int i0) __attribute__((always_inline)) {
            mask_below(x, (pre ? 0 : wkey0 + 32 * kc + lc) - i0 - 4 * lg);
            mask_above(x, S - 1 - i0 - 4 * lg);
        };
        u32x4 xf[2][2];
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) xf[kc][ks] = u32x4{0u, 0u, 0u, 0u};
        bf16x8 qa[8], ta[6];
        f32x16 nl, nl_n;
        f32x16 xa[2], xb[2];

        // The last two transposed fragments have a spare register set each (tb6 / tb7, indexed by
        // the parity of the iteration that USES them), so that the next iteration's copies can be
        // requested before this iteration's last use: nothing is issued to LDS in the last
        // groups, and the wait in front of the barrier finds (almost) nothing outstanding.
        bf16x8 tb6[2], tb7[2];
        auto stage = [&](auto hb_tag, auto masked_tag, int i0, f32x16 (&xin)[2], f32x16 (&xout)[2], const TileSrc& ts,
                         uint32_t wslot) __attribute__((always_inline)) {
            constexpr int hb = decltype(hb_tag)::value;
            constexpr bool MASKED = decltype(masked_tag)::value;
            if (MASKED) { mask1(xin[0], 0, i0 + 32 * hb); mask1(xin[1], 1, i0 + 32 * hb); }
            pin();
            float pe[32];
            u32x4 xn[2][2];
            auto elem = [&](int e) __attribute__((always_inline)) {
                pe[e] = fast_exp2(fmaf(xin[e >> 4][e & 15], c, nl[e & 15]));
            };
            auto pack2 = [&](int e) __attribute__((always_inline)) {     // elements e, e+1 -> their word of P(u)
                xn[e >> 4][(e & 15) >> 3][(e & 7) >> 1] = pack_bf16x2(pe[e], pe[e + 1]);
            };
            auto put = [&](int f) __attribute__((always_inline)) {       // fragment f of P(u) -> the pair's slot
                *(u32x4 __attribute__((address_space(3)))*)(wslot + f * 1024) = xn[f >> 1][f & 1];
            };
            static_for<32>([&](auto gc) __attribute__((always_inline)) {
                constexpr int g = decltype(gc)::value;
                if (g < 16) {
                    const int t8 = g >> 1, kc = g & 1;
                    if (t8 == 0) mma_vd_zero(xout[kc], qa[0], sf[kc][0]);
                    else         mma_vd(xout[kc], qa[t8], sf[kc][t8]);
                } else {
                    const int i = g - 16, ks = i >> 3, db = (i >> 1) & 3, kc = i & 1, pf = 4 * ks + db;
                    const bf16x8 tf = pf == 6 ? tb6[hb] : pf == 7 ? tb7[hb] : ta[pf];
                    acc[db][kc] = mma(tf, __builtin_bit_cast(bf16x8, xf[kc][ks]), acc[db][kc]);
                }
                __builtin_amdgcn_sched_barrier(0);   // the matrix-core instruction leads its group
                if (hb == 0 && g < KV_DMA0) dma_piece(ts, g);
                if (hb == 1 && g < KV_DMA - KV_DMA0) dma_piece(ts, KV_DMA0 + g);
                if (g == 20) ld_rows_at(nl_n, hb ? rofs : rofs_c, 1 - hb);                 // -lse2 of sub-tile u+1
                if (g >= 2 && g <= 16 && !(g & 1)) qa[(g - 2) >> 1] = ld_q((g - 2) >> 1, hb);   // of sub-tile u+2
                if (g >= 18 && g <= 28 && !(g & 1)) ta[(g - 18) >> 1] = ld_t((g - 18) >> 1, hb);   // of sub-tile u
                if (g == 25) tb6[1 - hb] = ld_t(6, hb);
                if (g == 27) tb7[1 - hb] = ld_t(7, hb);
                // P(u) leaves for the pair's slot fragment by fragment, as soon as each is complete
                if (g == 9) put(0);
                if (g == 17) put(1);
                if (g == 21) put(2);
                if (g == 29) put(3);
                __builtin_amdgcn_sched_barrier(0);   // LDS traffic first, then the vector ALU work
                // P(u): one element per group, two in groups 16-19, so that the last fragment is
                // complete four groups before the iteration ends
                if (g < 16) elem(g);
                else if (g < 20) { elem(2 * g - 16); elem(2 * g - 15); }
                else if (g < 28) elem(g + 4);
                if (g >= 2 && g <= 16 && !(g & 1)) pack2(g - 2);
                if (g >= 17 && g <= 20) pack2(2 * g - 18);
                if (g >= 22 && g <= 28 && !(g & 1)) pack2(g + 2);
                __builtin_amdgcn_sched_barrier(0);
            });
            nl = nl_n;
#pragma unroll
            for (int kc = 0; kc < 2; ++kc)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) xf[kc][ks] = xn[kc][ks];
            __builtin_amdgcn_sched_barrier(0);
        };
        auto settle = [&]() __attribute__((always_inline)) { asm volatile("s_nop 15\n\ts_nop 7" ::: "memory"); };

        int i0_cur, i0_nx;
        {   // prologue: tiles 0 and 1 on their way, scores of sub-tile 0, fragments of sub-tile 1
            const TileSrc t0s = next_tile(0);
            i0_cur = t0s.i0;
#pragma unroll
            for (int n = 0; n < KV_DMA; ++n) dma_piece(t0s, n);
            dma_wait();
            __syncthreads();
            const TileSrc t1s = next_tile(1);
            i0_nx = t1s.i0;
#pragma unroll
            for (int n = 0; n < KV_DMA; ++n) dma_piece(t1s, n);
#pragma unroll
            for (int t8 = 0; t8 < 8; ++t8) qa[t8] = lds_ld_frag(qofs[t8] - KV_BUF_B);        // sub-tile 0
            ld_rows_at(nl, rofs_c, 0);
#pragma unroll
            for (int t8 = 0; t8 < 8; ++t8) {
                if (t8 == 0) { mma_vd_zero(xa[0], qa[0], sf[0][0]); mma_vd_zero(xa[1], qa[0], sf[1][0]); }
                else         { mma_vd(xa[0], qa[t8], sf[0][t8]);    mma_vd(xa[1], qa[t8], sf[1][t8]); }
            }
            settle();
#pragma unroll
            for (int t8 = 0; t8 < 8; ++t8) qa[t8] = lds_ld_frag(qofs[t8] - KV_BUF_B + 32 * ROW_B);   // sub-tile 1
#pragma unroll
            for (int p = 0; p < 6; ++p) ta[p] = ld_t(p, 0);     // placeholder: multiplied by P = 0
            tb6[0] = ld_t(6, 0);
            tb7[0] = ld_t(7, 0);
        }
        int buf = 0;
        auto tile_iter = [&](auto masked_tag) __attribute__((always_inline)) {
            const int nbuf = buf + 1 == KV_NBUF ? 0 : buf + 1;
            const int nnbuf = nbuf + 1 == KV_NBUF ? 0 : nbuf + 1;
            const TileSrc ts = next_tile(nnbuf);
            dma_wait();       // tile T+1 has landed,
            lds_wait0();      // the last P went into its slot,
            wg_barrier();     // and everybody knows
            stage(std::integral_constant<int, 0>{}, masked_tag, i0_cur, xa, xb, ts, slot0);
            lds_wait0();
            wg_barrier();
            stage(std::integral_constant<int, 1>{}, masked_tag, i0_cur, xb, xa, ts, slot0 + KV_SLOT_B);
#pragma unroll
            for (int db = 0; db < 4; ++db) {                 // tile T -> T+1
                tofs[db][0] += nbuf == 0 ? back : fwd;
                tofs[db][1] += nbuf == 0 ? back : fwd;
            }
#pragma unroll
            for (int t8 = 0; t8 < 8; ++t8) qofs[t8] += nnbuf == 0 ? back : fwd;   // tile T+1 -> T+2
            rofs += nnbuf == 0 ? rback : rfwd;
            rofs_c += nbuf == 0 ? rback : rfwd;
            buf = nbuf;
            i0_cur = i0_nx;
            i0_nx = ts.i0;
        };
        for (int ti = 0; ti < nMain; ++ti) tile_iter(std::false_type{});
        for (int ti = nMain; ti < nT; ++ti) tile_iter(std::true_type{});
        __syncthreads();      // B's last iteration: publishes the last P
        {   // drain: the last sub-tile's contribution
            pin();
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const int pf = 4 * ks + db;
                    const bf16x8 tf = pf == 6 ? tb6[0] : pf == 7 ? tb7[0] : ta[pf];
                    acc[db][0] = mma(tf, __builtin_bit_cast(bf16x8, xf[0][ks]), acc[db][0]);
                    acc[db][1] = mma(tf, __builtin_bit_cast(bf16x8, xf[1][ks]), acc[db][1]);
                }
        }
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) {
            const int key = wkey0 + 32 * kc + lc;
            f32x16 col[4] = {acc[0][kc], acc[1][kc], acc[2][kc], acc[3][kc]};
            if (pre)
                kv_store_f32(col, key < P ? part_v + ((static_cast<size_t>(b) * Hkv + hk) * P + key) * HD : nullptr, lg, 1.f);
            else
                kv_store_bf16(col, key < S ? dv_own + ((t0 + key) * Hkv + hk) * HD : nullptr, lg, 1.f);
        }
    } else {
        // =========================================================================================
        // B: dP, dS, dK, one sub-tile behind A.  Iteration u: on entry yin = dP(u-1) - delta,
        // ga = row-wise dO fragments of sub-tile u, nd = -delta of sub-tile u, ta = transposed Q
        // fragments of sub-tile u-2, xf = dS(u-2); the slot of parity (u-1) holds P(u-1).
        // Matrix cores: dP(u) (groups 0-15), dK^T += Q^T dS(u-2) (groups 16-31); vector ALU:
        // dS(u-1) = P(u-1) (dP(u-1) - delta).
        // =========================================================================================
        uint32_t gofs[8], tofs[4][2], rofs;
        {
            const uint32_t tq0 = lds_addr(sm.t[0].q), tg0 = lds_addr(sm.t[0].g);
#pragma unroll
            for (int t8 = 0; t8 < 8; ++t8) gofs[t8] = tg0 + frag_n_ofs(lane, t8);
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                frag_t_ofs(lane, db, tofs[db][0], tofs[db][1]);
                tofs[db][0] += tq0;
                tofs[db][1] += tq0;
            }
            rofs = lds_addr(&sm.ndl[0][4 * lg]);
        }
        auto ld_g = [&](int t8, int half) __attribute__((always_inline)) { return lds_ld_frag(gofs[t8] + half * 32 * ROW_B); };
        auto ld_t = [&](int p, int half) __attribute__((always_inline)) {
            const int ks = p >> 2, db = p & 3;
            return lds_ld_frag_t(tofs[db][0] + (32 * half + 16 * ks) * ROW_B, tofs[db][1] + (32 * half + 16 * ks) * ROW_B);
        };
        auto ld_rows = [&](f32x16& d, int half) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const f32x4 w = lds_ld_f32x4(rofs + (32 * half + 8 * j) * 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) d[4 * j + e] = w[e];
            }
        };
        u32x4 xf[2][2];
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) xf[kc][ks] = u32x4{0u, 0u, 0u, 0u};
        bf16x8 ga[8], ta[8];
        f32x16 nd;
        f32x16 ya[2], yb[2];
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
            for (int r = 0; r < 16; ++r) ya[kc][r] = 0.f;      // "dP(-1)": multiplied by P(-1) = 0
        // P(-1) = 0 in the slot the first iteration reads (parity 1)
#pragma unroll
        for (int f = 0; f < 4; ++f)
            *(u32x4 __attribute__((address_space(3)))*)(slot0 + KV_SLOT_B + f * 1024) = u32x4{0u, 0u, 0u, 0u};

        // vector ALU part: dS(u-1) from the P fragments pw and yin; element e of 32
        auto ds_elem = [&](const u32x4 (&pw)[4], const f32x16 (&yin)[2], float (&w)[32], int e) __attribute__((always_inline)) {
            const int kc = e >> 4, r = e & 15;
            const uint32_t word = pw[2 * kc + (r >> 3)][(r & 7) >> 1];
            const float p = (r & 1) ? __uint_as_float(word & 0xffff0000u) : __uint_as_float(word << 16);
            w[e] = p * yin[kc][r];
        };
        // stage: `half` of the row-wise / row-value reads (sub-tile u+1) and `thalf` of the
        // transposed reads (sub-tile u-1) are fixed per call site
        auto stage = [&](auto hb_tag, f32x16 (&yin)[2], f32x16 (&yout)[2], uint32_t rslot) __attribute__((always_inline)) {
            constexpr int hb = decltype(hb_tag)::value;
            constexpr int half = 1 - hb;        // sub-tile u+1 is half 1 of tile T (hb 0) or half 0 of tile T+1 (hb 1)
            constexpr int thalf = 1 - hb;       // sub-tile u-1 is half 1 of tile T-1 (hb 0) or half 0 of tile T (hb 1)
            pin();
            u32x4 pw[4];
#pragma unroll
            for (int f = 0; f < 4; ++f) pw[f] = *(const u32x4 __attribute__((address_space(3)))*)(rslot + f * 1024);
            float w[32];
            u32x4 xn[2][2];
            static_for<32>([&](auto gc) __attribute__((always_inline)) {
                constexpr int g = decltype(gc)::value;
                if (g < 16) {
                    const int t8 = g >> 1, kc = g & 1;
                    if (t8 == 0) mma_vd_first(yout[kc], ga[0], sf[kc][0], nd);
                    else         mma_vd(yout[kc], ga[t8], sf[kc][t8]);
                } else {
                    const int i = g - 16, ks = i >> 3, db = (i >> 1) & 3, kc = i & 1;
                    acc[db][kc] = mma(ta[4 * ks + db], __builtin_bit_cast(bf16x8, xf[kc][ks]), acc[db][kc]);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (g == 20) ld_rows(nd, half);                                                   // -delta of sub-tile u+1
                if (g >= 2 && g <= 16 && !(g & 1)) ga[(g - 2) >> 1] = ld_g((g - 2) >> 1, half);   // of sub-tile u+1
                if (g >= 18 && !(g & 1)) ta[(g - 18) >> 1] = ld_t((g - 18) >> 1, thalf);          // of sub-tile u-1
                __builtin_amdgcn_sched_barrier(0);
                // dS(u-1): element g-4 from group 4 on (the P fragments were requested at the
                // top), the last four elements double up in the last four groups
                if (g >= 4) ds_elem(pw, yin, w, g - 4);
                if (g >= 28) ds_elem(pw, yin, w, g);
                if (g >= 6 && !(g & 1)) {
                    const int e = g - 6;
                    xn[e >> 4][(e & 15) >> 3][(e & 7) >> 1] = pack_bf16x2(w[e], w[e + 1]);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            ta[7] = ld_t(7, thalf);
            xn[1][1][1] = pack_bf16x2(w[26], w[27]);
            xn[1][1][2] = pack_bf16x2(w[28], w[29]);
            xn[1][1][3] = pack_bf16x2(w[30], w[31]);
#pragma unroll
            for (int kc = 0; kc < 2; ++kc)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) xf[kc][ks] = xn[kc][ks];
            __builtin_amdgcn_sched_barrier(0);
        };

        {   // prologue: A's barrier publishes tile 0; fragments and row values of sub-tile 0
            __syncthreads();
#pragma unroll
            for (int t8 = 0; t8 < 8; ++t8) ga[t8] = ld_g(t8, 0);
            ld_rows(nd, 0);
#pragma unroll
            for (int p = 0; p < 8; ++p) ta[p] = ld_t(p, 0);     // placeholder: multiplied by dS = 0
        }
        int buf = 0;
        bool first = true;
        auto tile_iter = [&]() __attribute__((always_inline)) {
            const int nbuf = buf + 1 == KV_NBUF ? 0 : buf + 1;
            const int nnbuf = nbuf + 1 == KV_NBUF ? 0 : nbuf + 1;
            wg_barrier();
            // first half: reads P of the previous tile's second sub-tile (parity 1)
            stage(std::integral_constant<int, 0>{}, ya, yb, slot0 + KV_SLOT_B);
            // between the halves the row-wise reads move on to tile T+1 and the transposed reads
            // to tile T (the first tile has no predecessor: they already sit on tile 0)
#pragma unroll
            for (int t8 = 0; t8 < 8; ++t8) gofs[t8] += nbuf == 0 ? back : fwd;
            rofs += nbuf == 0 ? rback : rfwd;
            if (!first) {
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    tofs[db][0] += buf == 0 ? back : fwd;
                    tofs[db][1] += buf == 0 ? back : fwd;
                }
            }
            wg_barrier();
            stage(std::integral_constant<int, 1>{}, yb, ya, slot0);
            first = false;
            buf = nbuf;
        };
        for (int ti = 0; ti < nT; ++ti) tile_iter();
        __syncthreads();
        {   // tail: dS of the last sub-tile, then the two outstanding dK products
            pin();
            u32x4 pw[4];
#pragma unroll
            for (int f = 0; f < 4; ++f) pw[f] = *(const u32x4 __attribute__((address_space(3)))*)(slot0 + KV_SLOT_B + f * 1024);
            // dK^T += Q^T dS(u-2): fragments of that sub-tile are in registers
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    acc[db][0] = mma(ta[4 * ks + db], __builtin_bit_cast(bf16x8, xf[0][ks]), acc[db][0]);
                    acc[db][1] = mma(ta[4 * ks + db], __builtin_bit_cast(bf16x8, xf[1][ks]), acc[db][1]);
                }
            float w[32];
#pragma unroll
            for (int e = 0; e < 32; ++e) ds_elem(pw, ya, w, e);
#pragma unroll
            for (int e = 0; e < 32; e += 2) xf[e >> 4][(e & 15) >> 3][(e & 7) >> 1] = pack_bf16x2(w[e], w[e + 1]);
            // the last sub-tile is the second half of the last tile, where the transposed reads sit
#pragma unroll
            for (int p = 0; p < 8; ++p) ta[p] = ld_t(p, 1);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    acc[db][0] = mma(ta[4 * ks + db], __builtin_bit_cast(bf16x8, xf[0][ks]), acc[db][0]);
                    acc[db][1] = mma(ta[4 * ks + db], __builtin_bit_cast(bf16x8, xf[1][ks]), acc[db][1]);
                }
        }
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) {
            const int key = wkey0 + 32 * kc + lc;
            f32x16 col[4] = {acc[0][kc], acc[1][kc], acc[2][kc], acc[3][kc]};
            if (pre)
                kv_store_f32(col, key < P ? part_k + ((static_cast<size_t>(b) * Hkv + hk) * P + key) * HD : nullptr, lg, scale);
            else
                kv_store_bf16(col, key < S ? dk_own + ((t0 + key) * Hkv + hk) * HD : nullptr, lg, scale);
        }
    }
}

__global__ __launch_bounds__(256, 1) void attn_bwd_kv_kernel(KvArgs args) {
#if defined(__HIP_DEVICE_COMPILE__)
    const KvArgs* ap = (const KvArgs*)__builtin_amdgcn_kernarg_segment_ptr();      // = &args
#else
    const KvArgs* ap = &args;
#endif
    // odd wavefronts take role B, even ones role A (wave-uniform: a scalar branch)
    if (__builtin_amdgcn_readfirstlane(threadIdx.x >> 6) & 1) kv_role<true>(ap);
    else                                                      kv_role<false>(ap);
}

// token rows per prefix-gradient partial, and the number of partials
int bwd_kv_chunk(const cart_attn_desc& d, long tokens, int* n_part) {
    const long nPb = (d.P + KV_WG_KEYS - 1) / KV_WG_KEYS;
    long n = nPb > 0 ? (KV_PREFIX_WGS + nPb * d.Hkv - 1) / (nPb * d.Hkv) : 1;
    const long most = (tokens + KV_MIN_CHUNK - 1) / KV_MIN_CHUNK;
    n = n < 1 ? 1 : (n > most ? most : n);
    const long chunk = (((tokens + n - 1) / n) + KV_TILE - 1) / KV_TILE * KV_TILE;
    *n_part = static_cast<int>((tokens + chunk - 1) / chunk);
    return static_cast<int>(chunk);
}

void launch_attn_bwd_kv(const cart_attn_desc& d, float scale, const bf16_t* Q, const bf16_t* K, const bf16_t* V,
                        const bf16_t* ZK, const bf16_t* ZV, const bf16_t* DO, const float* lse2, const float* delta,
                        bf16_t* dk, bf16_t* dv, float* part_k, float* part_v, const int32_t* cu, int n_tok, int chunk,
                        int n_part, hipStream_t st) {
    const long nPb = (d.P + KV_WG_KEYS - 1) / KV_WG_KEYS, nOb = (d.S + KV_WG_KEYS - 1) / KV_WG_KEYS;
    const unsigned grid = static_cast<unsigned>((nPb * n_part + nOb * d.B) * d.Hkv);
    KvArgs a;
    a.q = Q; a.k = K; a.v = V; a.zk = ZK; a.zv = ZV; a.d_o = DO; a.nlse2 = lse2; a.ndelta = delta;
    a.dk_own = dk; a.dv_own = dv; a.part_k = part_k; a.part_v = part_v; a.cu = cu;
    a.n_tok = n_tok; a.chunk = chunk; a.B = d.B; a.Smax = d.S; a.Hq = d.Hq; a.Hkv = d.Hkv; a.P = d.P;
    a.c = scale * CART_LOG2E; a.scale = scale;
    hipLaunchKernelGGL(attn_bwd_kv_kernel, dim3(grid), dim3(256), 0, st, a);
}

}  // namespace cart
