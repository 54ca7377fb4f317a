// Serve-time decode over a shared cartridge (Sec. 3.3; decode step of Sec. 2.3) on the matrix
// cores, bf16, head_dim 128.  One query token per request; keys = [prefix Z ; the request's own
// KV], all visible.
//
// The cartridge is shared by every request, so its part is a real GEMM: the B*G query rows
// that read one KV head (G = Hq/Hkv) are stacked and run against the prefix, split along the
// prefix into about half as many workgroups as there are CUs (prefix role).  The ragged own-KV
// part is bandwidth-bound: one wavefront per (request, KV head, chunk of keys) streams its chunk
// through a private LDS slot with the G query rows padded into one 32-column MFMA block (own
// role).  Both roles are workgroups of one launch (decode_fused_kernel), sized so that two share
// a CU: the matrix-core work on the L2-resident cartridge overlaps the HBM streaming of the own
// caches instead of preceding it.  Every split writes a normalised partial (O, lse);
// decode_merge_kernel combines them by their log-sum-exps.
//
// Composition (Sec. 5.4: cartridges trained apart are concatenated without retraining) and the
// per-request cartridges of App. A.3's serving protocol use the same two kernels: the shared
// prefix is a list of segments, each split and run like a single cartridge (a segment is never
// copied next to another), and a request's private cartridge is streamed like its own KV.
#include "attn_mfma.h"

namespace cart {
using namespace mfma;

constexpr int DEC_BM = 128;            // stacked query rows per prefix workgroup (4 x 32)
constexpr int DEC_BN = 32;             // prefix keys per LDS tile
constexpr int DEC_NBUF = 4;
// Prefix workgroups aimed at: half the CUs.  Measured on the serving shape (128 requests, 8192
// shared slots, own caches U[1,1024]): 64 -> 131 us, 128 -> 84 us, 192 -> 90 us, 256 -> 94 us,
// 512 -> 118 us for the whole call.
constexpr int DEC_PREFIX_WGS = 128;
constexpr int DEC_TILE_B = DEC_BN * ROW_B;
constexpr int DEC_SUB = 32;            // own keys per wavefront step
constexpr int DEC_SUB_B = DEC_SUB * ROW_B;

#ifndef DEC_OWN_CHUNK
#define DEC_OWN_CHUNK 256              // most keys per own / private-cartridge chunk of short caches
#endif
constexpr int DEC_MAX_SEG = CART_MAX_SEGMENTS;

// The shared prefix as a list of segments (one for a single cartridge), by value in the kernel
// arguments.  Segment s is split along its slots into n_ps[s] parts of tiles_per_split[s] tiles;
// its workgroups are blockIdx [blk0[s], blk0[s+1]) and its partial results slots slot0[s] + part.
struct PrefixTable {
    const bf16_t* zk[DEC_MAX_SEG];
    const bf16_t* zv[DEC_MAX_SEG];
    int p[DEC_MAX_SEG], tiles_per_split[DEC_MAX_SEG], n_ps[DEC_MAX_SEG], slot0[DEC_MAX_SEG];
    int blk0[DEC_MAX_SEG + 1];
    int n_seg;
};

struct DecodePlan {
    PrefixTable tab;
    int G, n_rb, n_ps;                    // prefix: row blocks, partial slots of all segments
    int chunk, n_cc, n_oc;                // keys per chunk; chunks of a private cartridge / own KV (worst case)
    size_t part_o_bytes, part_l_bytes;
};

// seg_p[n_seg]: slots per shared segment; pool_p: slots of a private cartridge (0 = none)
static DecodePlan make_plan(int B, int Hq, int Hkv, int max_own_len, const int* seg_p, int n_seg, int pool_p) {
    DecodePlan p;
    p.G = Hq / Hkv;
    const int rows = B * p.G;
    p.n_rb = (rows + DEC_BM - 1) / DEC_BM;
    int total_tiles = 0;
    for (int s = 0; s < n_seg; ++s) total_tiles += (seg_p[s] + DEC_BN - 1) / DEC_BN;
    int want = (DEC_PREFIX_WGS + Hkv * p.n_rb - 1) / (Hkv * p.n_rb);   // parts to reach that many workgroups
    want = want < 1 ? 1 : (want > total_tiles ? total_tiles : want);
    const int tps = total_tiles ? (total_tiles + want - 1) / want : 0;
    p.tab.n_seg = 0;
    p.tab.blk0[0] = 0;
    p.n_ps = 0;
    for (int s = 0; s < n_seg; ++s) {
        const int nPt = (seg_p[s] + DEC_BN - 1) / DEC_BN;
        if (nPt == 0) continue;                                     // an empty segment adds nothing
        const int k = p.tab.n_seg++;
        p.tab.p[k] = seg_p[s];
        p.tab.tiles_per_split[k] = tps;
        p.tab.n_ps[k] = (nPt + tps - 1) / tps;
        p.tab.slot0[k] = p.n_ps;
        p.n_ps += p.tab.n_ps[k];
        p.tab.blk0[k + 1] = p.tab.blk0[k] + Hkv * p.n_rb * p.tab.n_ps[k];
        p.tab.zk[k] = p.tab.zv[k] = nullptr;                        // filled by the launcher
    }
    p.chunk = (max_own_len > 4096 || pool_p > 4096) ? 1024 : DEC_OWN_CHUNK;
    p.n_cc = (pool_p + p.chunk - 1) / p.chunk;
    p.n_oc = (max_own_len + p.chunk - 1) / p.chunk;
    const size_t slots = static_cast<size_t>(p.n_ps + p.n_cc + p.n_oc) * B * Hq;
    p.part_o_bytes = (slots * HD * sizeof(float) + 255) & ~static_cast<size_t>(255);
    p.part_l_bytes = (slots * sizeof(float) + 255) & ~static_cast<size_t>(255);
    return p;
}

// Own rows of a request are split evenly over the n_oc chunk slots (in steps of 32 keys), so that
// every request keeps all its slots busy whatever its length: keys per chunk of a request.
__host__ __device__ __forceinline__ int own_chunk_keys(int len, int n_oc) {
    const int ck = ((len + n_oc - 1) / n_oc + DEC_SUB - 1) & ~(DEC_SUB - 1);
    return ck < DEC_SUB ? DEC_SUB : ck;
}

// Prefix role of the fused kernel: 128 stacked query rows (32 per wavefront) against one split of
// one segment, 32 keys per LDS tile, four tiles in rotation (tile u+1 feeds the next scores while
// tile u feeds O, tiles u+2 and u+3 are on their way).  Small on purpose -- at most 256 registers
// per lane and 64 KB of LDS -- so that two workgroups share a CU and the bandwidth-bound own-KV
// role runs beside it.  part_o [slot][B][Hq][128] fp32 (normalised), part_l [slot][B][Hq]
// (natural-log lse).
__device__ __forceinline__ void decode_prefix_role(char* sm, const bf16_t* __restrict__ q, const PrefixTable& tab,
                                                   float* __restrict__ part_o, float* __restrict__ part_l, int B,
                                                   int Hq, int Hkv, float c, int n_rb, int blk) {
    const int G = Hq / Hkv;
    int seg = 0;
    while (seg + 1 < tab.n_seg && blk >= tab.blk0[seg + 1]) ++seg;
    int id = blk - tab.blk0[seg];
    const int hk = id % Hkv; id /= Hkv;
    const int rb = id % n_rb;
    const int sp = id / n_rb;
    const bf16_t* zk = tab.zk[seg];
    const bf16_t* zv = tab.zv[seg];
    const int P = tab.p[seg], tiles_per_split = tab.tiles_per_split[seg];
    const int slot_base = tab.slot0[seg];
    const int lane = threadIdx.x & 63, lg = lane >> 5, lc = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rows = B * G;
    const int rho = rb * DEC_BM + 32 * wv + lc;

    bf16x8 qf[8];
    {
        const int rc = min(rho, rows - 1);
        const bf16_t* qp = q + (static_cast<size_t>(rc / G) * Hq + hk * G + rc % G) * HD + 8 * lg;
#pragma unroll
        for (int t = 0; t < 8; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(qp + 16 * t);
    }
    const int nPt = (P + DEC_BN - 1) / DEC_BN;
    const int t_lo = sp * tiles_per_split;
    const int nT = min(tiles_per_split, nPt - t_lo);
    const char* zk_b = reinterpret_cast<const char*>(zk) + static_cast<size_t>(hk) * P * ROW_B;
    const char* zv_b = reinterpret_cast<const char*>(zv) + static_cast<size_t>(hk) * P * ROW_B;
    char* smk = sm;
    char* smv = sm + DEC_NBUF * DEC_TILE_B;
    auto issue = [&](int t, int buf) __attribute__((always_inline)) {   // 2 + 2 loads per wavefront
        const int j0 = (t_lo + t) * DEC_BN;
        tile_load_async<DEC_BN>(smk + buf * DEC_TILE_B, zk_b, j0, P - 1, ROW_B);
        tile_load_async<DEC_BN>(smv + buf * DEC_TILE_B, zv_b, j0, P - 1, ROW_B);
    };

    f32x16 acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
    float m_run = NEG_BIG, l_run = 0.f;
    f32x16 s;
    auto scores = [&](const char* kt) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) s = mma(lds_frag_n(kt, lc, 16 * t8 + 8 * lg), qf[t8], s);
    };
    // mask the ragged end of the segment, then move the running maximum when the tile's exceeds
    // it by more than RESCALE_GAP (rare after the first tile)
    auto prepare = [&](int t, bool live) __attribute__((always_inline)) {
        const int j0 = (t_lo + t) * DEC_BN;
        if (live && j0 + DEC_BN > P) {
            const int thr = P - 1 - j0 - 4 * lg;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (8 * (r >> 2) + (r & 3) > thr) s[r] = NEG_BIG;
        }
        float tm = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) tm = fmaxf(tm, s[r]);
        tm = partner_max(tm) * c;
        const float m_new = (live && tm > m_run + RESCALE_GAP) ? tm : m_run;
        if (__any(m_new != m_run)) {
            const float alpha = fast_exp2(m_run - m_new);
            l_run *= alpha;
            m_run = m_new;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[db][r] *= alpha;
        }
    };

    issue(0, 0);
    issue(min(1, nT - 1), 1);
    issue(min(2, nT - 1), 2);
    dma_wait_but<8>();          // tile 0
    __syncthreads();
    scores(smk);
    prepare(0, true);
    for (int u = 0; u < nT; ++u) {
        const int buf = u & 3;
        float rs = 0.f;
        f32x16 p;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            p[r] = fast_exp2(fmaf(s[r], c, -m_run));
            rs += p[r];
        }
        l_run += rs;
        const bf16x8 pf0 = pack_frag(p, 0), pf1 = pack_frag(p, 8);
        // tile u+1 has landed for every wavefront and tile u-1 is no longer read: its buffer
        // takes tile u+3 (past the end the last tile again, into a buffer nobody reads)
        dma_wait_but<4>();
        __syncthreads();
        issue(min(u + 3, nT - 1), (u + 3) & 3);
        if (u + 1 < nT) scores(smk + ((u + 1) & 3) * DEC_TILE_B);
        const char* vt = smv + buf * DEC_TILE_B;
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            acc[db] = mma(lds_frag_t(vt, 0, 32 * db, lane), pf0, acc[db]);
            acc[db] = mma(lds_frag_t(vt, 16, 32 * db, lane), pf1, acc[db]);
        }
        prepare(u + 1, u + 1 < nT);
    }
    dma_wait();
    const float l_tot = l_run + partner(l_run);
    const float inv = 1.f / l_tot;
    if (rho < rows) {
        const size_t slot = (static_cast<size_t>(slot_base + sp) * B + rho / G) * Hq + hk * G + rho % G;
        float* op = part_o + slot * HD;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                typedef float f32x4 __attribute__((ext_vector_type(4)));
                f32x4 w = {acc[db][4 * r4] * inv, acc[db][4 * r4 + 1] * inv, acc[db][4 * r4 + 2] * inv,
                           acc[db][4 * r4 + 3] * inv};
                *reinterpret_cast<f32x4*>(op + 32 * db + 8 * r4 + 4 * lg) = w;
            }
        if (lg == 0) part_l[slot] = (m_run + fast_log2(l_tot)) * CART_LN2;
    }
}

// One wavefront per (request, KV head, chunk of keys): chunks 0 .. n_cc-1 cover the request's
// private cartridge pool[cart_id[b]] ([Hkv,pool_p,128]; none when cart_id is null or negative),
// chunks n_cc .. n_cc+n_oc-1 its own KV rows, split evenly over those slots.  32 keys per step through a private 16 KB LDS
// slot; the G query rows of the group occupy columns 0..G-1 of one MFMA block.
__device__ __forceinline__ void decode_own_role(
    char* sm /* [wavefront][K, V][32 rows] */, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
    const bf16_t* __restrict__ v, const int32_t* __restrict__ cu, const bf16_t* __restrict__ pool_k,
    const bf16_t* __restrict__ pool_v, const int32_t* __restrict__ cart_id, int pool_p,
    float* __restrict__ part_o, float* __restrict__ part_l, int B, int Hq, int Hkv, float c, int chunk, int n_cc,
    int n_oc, int n_ps, int blk) {
    const int G = Hq / Hkv;
    const int lane = threadIdx.x & 63, lg = lane >> 5, lc = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    long item = static_cast<long>(blk) * 4 + wv;
    const int hk = item % Hkv; item /= Hkv;
    const int cc = item % (n_cc + n_oc);
    const int b = static_cast<int>(item / (n_cc + n_oc));
    if (b >= B) return;
    const bool priv = cc < n_cc;
    int len, k0, ck = chunk;
    uint32_t pitch;
    const char *k_b, *v_b;
    if (priv) {
        const int cid = cart_id ? cart_id[b] : -1;
        if (cid < 0) return;
        len = pool_p;
        k0 = cc * chunk;
        pitch = ROW_B;
        const size_t row0 = (static_cast<size_t>(cid) * Hkv + hk) * pool_p + k0;
        k_b = reinterpret_cast<const char*>(pool_k) + row0 * ROW_B;
        v_b = reinterpret_cast<const char*>(pool_v) + row0 * ROW_B;
    } else {
        const int t0 = cu[b];
        len = cu[b + 1] - t0;
        ck = own_chunk_keys(len, n_oc);
        k0 = (cc - n_cc) * ck;
        pitch = static_cast<uint32_t>(Hkv) * ROW_B;
        const size_t row0 = static_cast<size_t>(t0 + k0) * Hkv + hk;
        k_b = reinterpret_cast<const char*>(k) + row0 * ROW_B;
        v_b = reinterpret_cast<const char*>(v) + row0 * ROW_B;
    }
    if (k0 >= len) return;
    const int nk = min(ck, len - k0);

    bf16x8 qf[8];
    {
        const bf16_t* qp = q + (static_cast<size_t>(b) * Hq + hk * G + min(lc, G - 1)) * HD + 8 * lg;
#pragma unroll
        for (int t = 0; t < 8; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(qp + 16 * t);
    }
    char* kt = sm + (2 * wv) * DEC_SUB_B;
    char* vt = kt + DEC_SUB_B;
    // 32 rows x 256 B = 8 direct-to-LDS loads of 4 rows each, per tensor, by this wavefront alone
    auto issue = [&](int j0) __attribute__((always_inline)) {
        const size_t step = static_cast<size_t>(j0) * pitch;
        const int lim = nk - 1 - j0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int r = 4 * i + (lane >> 4);
            const uint32_t off = static_cast<uint32_t>(min(r, lim)) * pitch + (((lane & 15) ^ swz(r)) << 4);
            dma16(k_b + step, off, lds_addr(kt) + 4 * i * ROW_B);
            dma16(v_b + step, off, lds_addr(vt) + 4 * i * ROW_B);
        }
    };

    f32x16 acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
    float m_run = NEG_BIG, l_run = 0.f;
    issue(0);
    for (int j0 = 0; j0 < nk; j0 += DEC_SUB) {
        // fragments of this step into registers, then the next step's loads overwrite the slot
        // while the matrix cores work
        bf16x8 ka[8], va[2][4];
        dma_wait();   // this step's direct-to-LDS loads have landed
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) ka[t8] = lds_frag_n(kt, lc, 16 * t8 + 8 * lg);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) va[ks][db] = lds_frag_t(vt, 16 * ks, 32 * db, lane);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (j0 + DEC_SUB < nk) issue(j0 + DEC_SUB);
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) s = mma(ka[t8], qf[t8], s);
        if (j0 + DEC_SUB > nk) {
            const int thr = nk - 1 - j0 - 4 * lg;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (8 * (r >> 2) + (r & 3) > thr) s[r] = NEG_BIG;
        }
        float tm = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) tm = fmaxf(tm, s[r]);
        tm = partner_max(tm) * c;
        const float m_new = fmaxf(m_run, tm);
        const float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;
        float rs = 0.f;
        f32x16 p;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            p[r] = fast_exp2(fmaf(s[r], c, -m_run));
            rs += p[r];
        }
        l_run = l_run * alpha + rs;
        const bf16x8 pf0 = pack_frag(p, 0), pf1 = pack_frag(p, 8);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] *= alpha;
            acc[db] = mma(va[0][db], pf0, acc[db]);
            acc[db] = mma(va[1][db], pf1, acc[db]);
        }
    }
    const float l_tot = l_run + partner(l_run);
    const float inv = 1.f / l_tot;
    if (lc < G) {
        const size_t slot = (static_cast<size_t>(n_ps + cc) * B + b) * Hq + hk * G + lc;
        float* op = part_o + slot * HD;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                typedef float f32x4 __attribute__((ext_vector_type(4)));
                f32x4 w = {acc[db][4 * r4] * inv, acc[db][4 * r4 + 1] * inv, acc[db][4 * r4 + 2] * inv,
                           acc[db][4 * r4 + 3] * inv};
                *reinterpret_cast<f32x4*>(op + 32 * db + 8 * r4 + 4 * lg) = w;
            }
        if (lg == 0) part_l[slot] = (m_run + fast_log2(l_tot)) * CART_LN2;
    }
}

// Both roles in one launch, two workgroups per CU: prefix workgroups (matrix-core and LDS work
// on data that sits in L2) and own-KV workgroups (HBM streaming) alternate in the grid while
// both kinds remain, so that the two run side by side instead of one after the other.
__global__ __launch_bounds__(256, 2) void decode_fused_kernel(
    const bf16_t* __restrict__ q, const PrefixTable tab, const bf16_t* __restrict__ k,
    const bf16_t* __restrict__ v, const int32_t* __restrict__ cu, const bf16_t* __restrict__ pool_k,
    const bf16_t* __restrict__ pool_v, const int32_t* __restrict__ cart_id, int pool_p,
    float* __restrict__ part_o, float* __restrict__ part_l, int B, int Hq, int Hkv, float c, int n_rb, int chunk,
    int n_cc, int n_oc, int n_ps, int n_pre_wg, int n_own_wg) {
    static_assert(2 * DEC_NBUF * DEC_TILE_B == 4 * 2 * DEC_SUB_B, "the two roles share one LDS block");
    __shared__ __attribute__((aligned(16))) char sm[4 * 2 * DEC_SUB_B];
    const int i = blockIdx.x;
    const int both = min(n_pre_wg, n_own_wg);
    bool pre;
    int idx;
    // The roles alternate in runs of 8 workgroups (consecutive workgroups go to the 8 XCDs in
    // turn): every XCD hosts both roles, and with 8 KV heads a prefix workgroup's head
    // (idx % Hkv) is its XCD, whose L2 then holds that one head's cartridge.
    const int both8 = both & ~7;
    if (i < 2 * both8) { pre = !((i >> 3) & 1); idx = ((i >> 4) << 3) | (i & 7); }
    else               { const int r = i - 2 * both8, left = both - both8;
                         if (r < 2 * left) { pre = !(r & 1); idx = both8 + (r >> 1); }
                         else              { pre = n_pre_wg > n_own_wg; idx = i - both; } }
    if (pre) decode_prefix_role(sm, q, tab, part_o, part_l, B, Hq, Hkv, c, n_rb, idx);
    else     decode_own_role(sm, q, k, v, cu, pool_k, pool_v, cart_id, pool_p, part_o, part_l, B, Hq, Hkv, c, chunk,
                             n_cc, n_oc, n_ps, idx);
}

// o[b,h,:] = sum_i w_i part_o[i] / sum_i w_i, w_i = exp(lse_i - max lse), over the partial slots
// that exist for the request: the n_ps prefix parts, the chunks of its private cartridge (when it
// has one), the chunks of its own rows (own_chunk_keys(len) keys each).  One wavefront per
// (b, h), the slots in groups of 64: lane i holds the lse and the weight of the group's slot i,
// then every lane accumulates its two head elements over the group's slots with the loads of
// eight slots in flight.
__global__ __launch_bounds__(256) void decode_merge_kernel(const float* __restrict__ part_o,
                                                           const float* __restrict__ part_l,
                                                           const int32_t* __restrict__ cu,
                                                           const int32_t* __restrict__ cart_id, int pool_p,
                                                           bf16_t* __restrict__ o,
                                                           float* __restrict__ lse, int B, int Hq,
                                                           int n_ps, int n_cc, int n_oc, int chunk) {
    const int lane = threadIdx.x & 63;
    const long row = static_cast<long>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (row >= static_cast<long>(B) * Hq) return;
    const int b = row / Hq;
    const int len = cu[b + 1] - cu[b];
    const int priv = (n_cc > 0 && cart_id && cart_id[b] >= 0) ? (pool_p + chunk - 1) / chunk : 0;
    const int ck = own_chunk_keys(len, n_oc);
    const int own = (len + ck - 1) / ck;
    const int n = n_ps + n_cc + n_oc;
    auto valid = [&](int i) { return i < n_ps || (i < n_ps + n_cc ? i - n_ps < priv : i - n_ps - n_cc < own); };
    const size_t stride = static_cast<size_t>(B) * Hq;
    // slots in groups of 64: lane i holds the lse and the weight of slot g0 + i
    float m = -3.0e38f;
    for (int g0 = 0; g0 < n; g0 += 64) {
        const int i = g0 + lane;
        if (i < n && valid(i)) m = fmaxf(m, part_l[i * stride + row]);
    }
    m = wave_max(m);
    float wsum = 0.f, a0 = 0.f, a1 = 0.f;
    for (int g0 = 0; g0 < n; g0 += 64) {
        const int cnt = min(64, n - g0);
        const bool mine = lane < cnt && valid(g0 + lane);
        const float wi = mine ? __expf(part_l[(g0 + lane) * stride + row] - m) : 0.f;
        wsum += wi;
        int i = 0;
        for (; i + 8 <= cnt; i += 8) {
            float2 x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                x[j] = float2{0.f, 0.f};
                if (valid(g0 + i + j))
                    x[j] = *reinterpret_cast<const float2*>(part_o + ((g0 + i + j) * stride + row) * HD + 2 * lane);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float w = __shfl(wi, i + j);
                a0 = fmaf(w, x[j].x, a0);
                a1 = fmaf(w, x[j].y, a1);
            }
        }
        for (; i < cnt; ++i) {
            if (!valid(g0 + i)) continue;
            const float w = __shfl(wi, i);
            const float2 x = *reinterpret_cast<const float2*>(part_o + ((g0 + i) * stride + row) * HD + 2 * lane);
            a0 = fmaf(w, x.x, a0);
            a1 = fmaf(w, x.y, a1);
        }
    }
    wsum = wave_sum(wsum);
    const float inv = 1.f / wsum;
    *reinterpret_cast<uint32_t*>(o + row * HD + 2 * lane) = pack_bf16x2(a0 * inv, a1 * inv);
    if (lane == 0 && lse) lse[row] = m + __logf(wsum);
}

bool decode_mfma_supported(const cart_decode_desc& d) {
    return d.dtype == CART_BF16 && d.D == 128 && d.Hq / d.Hkv <= 32;
}

size_t decode_mfma_workspace(const cart_decode_desc& d) {
    const DecodePlan p = make_plan(d.B, d.Hq, d.Hkv, d.max_own_len, &d.P, d.P > 0 ? 1 : 0, 0);
    return p.part_o_bytes + p.part_l_bytes;
}

bool decode_composed_supported(const cart_decode_composed_desc& d) {
    return d.dtype == CART_BF16 && d.D == 128 && d.Hq / d.Hkv <= 32;
}

static DecodePlan composed_plan(const cart_decode_composed_desc& d, const cart_segment* shared) {
    int seg_p[DEC_MAX_SEG];
    for (int s = 0; s < d.n_shared; ++s) seg_p[s] = shared[s].p;
    return make_plan(d.B, d.Hq, d.Hkv, d.max_own_len, seg_p, d.n_shared, d.n_pool > 0 ? d.pool_p : 0);
}

size_t decode_composed_workspace(const cart_decode_composed_desc& d, const cart_segment* shared) {
    const DecodePlan p = composed_plan(d, shared);
    return p.part_o_bytes + p.part_l_bytes;
}

// prefix parts, then private-cartridge and own chunks, then the merge
static int run_decode(const DecodePlan& p, int B, int Hq, int Hkv, float scale, const void* q, const void* pool_k,
                      const void* pool_v, const int32_t* cart_id, int pool_p, const void* k, const void* v,
                      const int32_t* cu, void* o, float* lse, void* ws, hipStream_t st) {
    float* part_o = static_cast<float*>(ws);
    float* part_l = reinterpret_cast<float*>(static_cast<char*>(ws) + p.part_o_bytes);
    const float c = scale * CART_LOG2E;
    const long items = static_cast<long>(B) * Hkv * (p.n_cc + p.n_oc);
    const int n_own_wg = static_cast<int>((items + 3) / 4);
    const bf16_t *Q = static_cast<const bf16_t*>(q), *K = static_cast<const bf16_t*>(k), *V = static_cast<const bf16_t*>(v),
                 *PK = static_cast<const bf16_t*>(pool_k), *PV = static_cast<const bf16_t*>(pool_v);
    trace_begin(st);   // kernel order: prefix + own (one launch), merge
    const int n_pre_wg = p.n_ps > 0 ? p.tab.blk0[p.tab.n_seg] : 0;
    hipLaunchKernelGGL(decode_fused_kernel, dim3(static_cast<unsigned>(n_pre_wg + n_own_wg)), dim3(256), 0, st, Q, p.tab,
                       K, V, cu, PK, PV, cart_id, pool_p, part_o, part_l, B, Hq, Hkv, c, p.n_rb, p.chunk, p.n_cc,
                       p.n_oc, p.n_ps, n_pre_wg, n_own_wg);
    trace_mark(st);
    const long rows = static_cast<long>(B) * Hq;
    hipLaunchKernelGGL(decode_merge_kernel, dim3(static_cast<unsigned>((rows + 3) / 4)), dim3(256), 0, st, part_o,
                       part_l, cu, cart_id, pool_p, static_cast<bf16_t*>(o), lse, B, Hq, p.n_ps, p.n_cc, p.n_oc,
                       p.chunk);
    trace_mark(st);
    return static_cast<int>(hipGetLastError());
}

int launch_decode_mfma(const cart_decode_desc& d, float scale, const void* q, const void* zk,
                       const void* zv, const void* k, const void* v, const int32_t* cu, void* o,
                       float* lse, void* ws, hipStream_t st) {
    DecodePlan p = make_plan(d.B, d.Hq, d.Hkv, d.max_own_len, &d.P, d.P > 0 ? 1 : 0, 0);
    if (p.tab.n_seg > 0) {
        p.tab.zk[0] = static_cast<const bf16_t*>(zk);
        p.tab.zv[0] = static_cast<const bf16_t*>(zv);
    }
    return run_decode(p, d.B, d.Hq, d.Hkv, scale, q, nullptr, nullptr, nullptr, 0, k, v, cu, o, lse, ws, st);
}

// ---- the decode step for callers that cannot allocate ---------------------------------------------
// The partial results of one call live in a file-scope device array instead of a caller-supplied
// workspace.  Each GPU holds its own copy of the array at its own address, looked up once per
// device; host code only ever uses that looked-up address, never the array's name.
constexpr size_t DEC_STATIC_BYTES = static_cast<size_t>(32) << 20;
static __device__ __align__(256) unsigned char scratch[DEC_STATIC_BYTES];
constexpr int DEC_MAX_DEVICES = 64;
static void* g_scratch_ptr[DEC_MAX_DEVICES];      // per device, nullptr until looked up

size_t decode_static_capacity() { return DEC_STATIC_BYTES; }

// the current device's copy of the array (nullptr when the runtime refuses the lookup)
void* decode_static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= DEC_MAX_DEVICES) return nullptr;
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

int launch_decode_composed(const cart_decode_composed_desc& d, float scale, const void* q,
                           const cart_segment* shared, const void* pool_k, const void* pool_v,
                           const int32_t* cart_id, const void* k, const void* v, const int32_t* cu, void* o,
                           float* lse, void* ws, hipStream_t st) {
    DecodePlan p = composed_plan(d, shared);
    int kseg = 0;
    for (int s = 0; s < d.n_shared; ++s) {
        if (shared[s].p <= 0) continue;
        p.tab.zk[kseg] = static_cast<const bf16_t*>(shared[s].z_k);
        p.tab.zv[kseg] = static_cast<const bf16_t*>(shared[s].z_v);
        ++kseg;
    }
    const bool pool = d.n_pool > 0 && d.pool_p > 0;
    return run_decode(p, d.B, d.Hq, d.Hkv, scale, q, pool ? pool_k : nullptr, pool ? pool_v : nullptr,
                      pool ? cart_id : nullptr, pool ? d.pool_p : 0, k, v, cu, o, lse, ws, st);
}

}  // namespace cart
