// Serve-time decode over a shared cartridge (Sec. 3.3; decode step of Sec. 2.3) on the matrix
// cores, bf16, head_dim 128.  One query token per request; keys = [prefix Z ; the request's own
// KV], all visible.
//
// The cartridge is shared by every request, so its part is a real GEMM: the B*G query rows
// that read one KV head (G = Hq/Hkv) are stacked and run against the prefix, split along the
// prefix into workgroups of 128 rows (prefix role).  The ragged own-KV part is bandwidth-bound:
// the packed own caches are cut evenly along their token axis, whatever the requests' lengths,
// and every resident wavefront streams one range of one KV head through a private LDS slot, with
// the G query rows of the request it is passing padded into one 32-column MFMA block (own role).
// Both roles are workgroups of one launch (decode_fused_kernel), sized so that two share a CU --
// the matrix-core work on the L2-resident cartridge overlaps the HBM streaming of the own caches
// instead of preceding it -- and the launch holds no more workgroups than the chip keeps
// resident.  Every split writes a normalised partial (O, lse); decode_merge_kernel combines them
// by their log-sum-exps.
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
#ifndef DEC_NBUF
#define DEC_NBUF 4                     // prefix tiles in LDS: one read, one ready, the rest in flight
#endif
// Prefix workgroups aimed at.  Measured on the serving shape (128 requests, 8192 shared slots,
// own caches U[1,1024]), fused kernel + merge: 96 -> 66.8 + 7.6 us, 128 -> 57.7 + 8.0, 160 ->
// 59.3 + 8.8, 192 -> 53.0 + 9.0, 256 -> 60.8 + 10.0.  The prefix workgroups and the own-KV
// workgroups that share their CUs are the last to finish; more, shorter prefix workgroups end
// closer to the rest, until their extra partials cost more in the merge.
constexpr int DEC_PREFIX_WGS = 192;
constexpr int DEC_TILE_B = DEC_BN * ROW_B;
constexpr int DEC_SUB = 32;            // own keys per wavefront step
constexpr int DEC_SUB_B = DEC_SUB * ROW_B;

#ifndef DEC_POOL_CHUNK
#define DEC_POOL_CHUNK 256             // fewest keys per chunk of a private cartridge
#endif
constexpr int DEC_MIN_SHARE = 256;      // fewest token rows per own-KV range (a multiple of DEC_SUB)
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
    int chunk, n_cc;                      // private cartridge: keys per chunk, chunks
    int share, n_oc, n_own_wg;            // own KV: token rows per range, most ranges a request reaches into, workgroups
    size_t part_o_bytes, part_l_bytes;
};

// workgroups of 256 threads the chip holds at two per CU (per device, looked up once)
static int resident_wgs() {
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 512;
    if (!cached[dev]) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        cached[dev] = 2 * cus;
    }
    return cached[dev];
}

// seg_p[n_seg]: slots per shared segment; pool_p: slots of a private cartridge (0 = none);
// T: rows of the packed own caches
static DecodePlan make_plan(int B, int Hq, int Hkv, int max_own_len, int T, const int* seg_p, int n_seg, int pool_p) {
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
    // Own KV: the workgroups that stay resident beside the prefix workgroups, four wavefronts
    // each, one wavefront per (range of token rows, KV head); the ranges cut T evenly, in whole
    // steps of 32 rows.
    const int n_pre_wg = p.n_ps > 0 ? p.tab.blk0[p.tab.n_seg] : 0;
    long wgs = resident_wgs() - n_pre_wg;
    if (wgs < 64) wgs = 64;
    long ranges = 4 * wgs / Hkv;
    if (ranges < 1) { ranges = 1; wgs = (Hkv + 3) / 4; }
    // (not below DEC_MIN_SHARE rows: shorter ranges only multiply the partials a request leaves)
    long share = ((static_cast<long>(T) + ranges - 1) / ranges + DEC_SUB - 1) / DEC_SUB * DEC_SUB;
    if (share < DEC_MIN_SHARE) share = DEC_MIN_SHARE;
    const long used = (static_cast<long>(T) + share - 1) / share;            // ranges that hold rows
    if (pool_p == 0 && (used * Hkv + 3) / 4 < wgs) wgs = (used * Hkv + 3) / 4;
    // Private cartridges: chunks sized so that there is about one per wavefront (measured on 128
    // requests x 2048 slots: chunks of 256 / 512 / 1024 / 2048 slots -> 0.268 / 0.259 / 0.254 /
    // 0.248 ms: every chunk starts with a round trip nothing overlaps), not below DEC_POOL_CHUNK
    p.chunk = DEC_POOL_CHUNK;
    if (pool_p > 0) {
        const long rows = static_cast<long>(B) * Hkv * pool_p;
        long ck = ((rows + 4 * wgs - 1) / (4 * wgs) + DEC_SUB - 1) / DEC_SUB * DEC_SUB;
        const long whole = (static_cast<long>(pool_p) + DEC_SUB - 1) / DEC_SUB * DEC_SUB;
        if (ck < DEC_POOL_CHUNK) ck = DEC_POOL_CHUNK;
        if (ck > whole) ck = whole;
        p.chunk = static_cast<int>(ck);
    }
    p.n_cc = (pool_p + p.chunk - 1) / p.chunk;
    p.share = static_cast<int>(share);
    p.n_own_wg = static_cast<int>(wgs);
    p.n_oc = static_cast<int>((max_own_len + share - 1) / share) + 1;
    const size_t slots = static_cast<size_t>(p.n_ps + p.n_cc + p.n_oc) * B * Hq;
    p.part_o_bytes = (slots * HD * sizeof(float) + 255) & ~static_cast<size_t>(255);
    p.part_l_bytes = (slots * sizeof(float) + 255) & ~static_cast<size_t>(255);
    return p;
}

// Prefix role of the fused kernel: 128 stacked query rows (32 per wavefront) against one split of
// one segment, 32 keys per LDS tile, DEC_NBUF tiles in rotation.  Small on purpose -- at most 256 registers
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
    // entries past the last slot of the segment, in the scores of tile t
    auto mask_tail = [&](int t) __attribute__((always_inline)) {
        const int j0 = (t_lo + t) * DEC_BN;
        if (j0 + DEC_BN > P) {
            const int thr = P - 1 - j0 - 4 * lg;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (8 * (r >> 2) + (r & 3) > thr) s[r] = NEG_BIG;
        }
    };
    // largest scaled score of the tile in s, over both halves of the lane's row
    auto row_max = [&]() __attribute__((always_inline)) {
        float tm = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) tm = fmaxf(tm, s[r]);
        return partner_max(tm) * c;
    };

    // Pipeline.  Entering iteration u a wavefront holds, in registers, the masked scores of tile
    // u, the K fragments of tile u+1 and the V fragments of tile u.  The iteration issues the 8
    // score products of tile u+1 and the 8 O products of tile u; each fragment register is
    // refilled from LDS right behind the product that consumed it (K of tile u+2, V of tile u+1),
    // and the exponentials of tile u run between the score products.  Requested all together
    // behind the barrier instead, the four wavefronts' 64 KB of fragment reads per tile keep LDS
    // busy for as long as the products keep the matrix cores busy, one after the other.
    //   What bounds an iteration is the number of instructions the one wavefront of a SIMD has to
    // issue besides its 16 products (measured 0.74 us per tile against 0.25 us of products with
    // about 250 of them), so everything that is not per-element work is kept out of the loop:
    //   - the loop is unrolled over the DEC_NBUF buffers, which makes every LDS address of an
    //     iteration a per-lane constant plus an immediate;
    //   - the softmax reference m is the maximum of the FIRST tile and is not looked for again:
    //     the exponentials are formed against it, and only if a lane's row sum for the tile
    //     exceeds 2^12 -- some score lies more than 2^8 above m, or the sum has overflowed -- does
    //     the wavefront take the tile's true maximum, rescale O and l, and form the tile's
    //     exponentials again.  A false alarm costs time, not accuracy.
    // Buffers: tiles u+1 and u+2 are read, tile u+3 is in flight, the buffer of tile u is free
    // once every wavefront's reads of it have completed -- the wait and the barrier at the top --
    // and takes tile u+4.  Past the end of the split the last tile is requested again and stale
    // buffers are read; nothing formed from them is used.
    static_assert(DEC_NBUF == 4, "the rotation below is written for four buffers");
    constexpr float OVER = 4096.f;
#pragma unroll
    for (int t = 0; t < DEC_NBUF; ++t) issue(min(t, nT - 1), t);
    dma_wait_but<4 * (DEC_NBUF - 2)>();          // tiles 0 and 1
    __syncthreads();
    scores(smk);
    mask_tail(0);
    m_run = row_max();
    bf16x8 ka[8], va[2][4];
#pragma unroll
    for (int t8 = 0; t8 < 8; ++t8) ka[t8] = lds_frag_n(smk + DEC_TILE_B, lc, 16 * t8 + 8 * lg);
#pragma unroll
    for (int db = 0; db < 4; ++db) {
        va[0][db] = lds_frag_t(smv, 0, 32 * db, lane);
        va[1][db] = lds_frag_t(smv, 16, 32 * db, lane);
    }
    auto body = [&](auto buf_c, int u) __attribute__((always_inline)) {
        constexpr int BUF = decltype(buf_c)::value;
        dma_wait_but<4 * (DEC_NBUF - 3)>();       // tile u+2
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __syncthreads();
        issue(min(u + DEC_NBUF, nT - 1), BUF);
        const char* kn = smk + ((BUF + 2) % DEC_NBUF) * DEC_TILE_B;
        const char* vn = smv + ((BUF + 1) % DEC_NBUF) * DEC_TILE_B;
        f32x16 sn;
        uint32_t pw[8];
        float rs = 0.f;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) {
            // written out so that the product stays in this place: the compiler is free to move
            // the builtin across the fences, and gathers all eight at the end of the iteration.
            // sn is next read by vector instructions behind the eight O products.
            if (t8 == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(sn) : "v"(ka[0]), "v"(qf[0]));
            else         asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(sn) : "v"(ka[t8]), "v"(qf[t8]));
            ka[t8] = lds_frag_n(kn, lc, 16 * t8 + 8 * lg);
            const float p0 = fast_exp2(fmaf(s[2 * t8], c, -m_run));
            const float p1 = fast_exp2(fmaf(s[2 * t8 + 1], c, -m_run));
            rs += p0;
            rs += p1;
            pw[t8] = pack_bf16x2(p0, p1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (__any(!(rs <= OVER))) {
            const float m_new = fmaxf(m_run, row_max());
            const float alpha = fast_exp2(m_run - m_new);
            l_run *= alpha;
            m_run = m_new;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[db][r] *= alpha;
            rs = 0.f;
#pragma unroll
            for (int t8 = 0; t8 < 8; ++t8) {
                const float p0 = fast_exp2(fmaf(s[2 * t8], c, -m_run));
                const float p1 = fast_exp2(fmaf(s[2 * t8 + 1], c, -m_run));
                rs += p0 + p1;
                pw[t8] = pack_bf16x2(p0, p1);
            }
        }
        l_run += rs;
        const bf16x8 pf0 = __builtin_bit_cast(bf16x8, u32x4{pw[0], pw[1], pw[2], pw[3]});
        const bf16x8 pf1 = __builtin_bit_cast(bf16x8, u32x4{pw[4], pw[5], pw[6], pw[7]});
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            acc[db] = mma(va[0][db], pf0, acc[db]);
            va[0][db] = lds_frag_t(vn, 0, 32 * db, lane);
            __builtin_amdgcn_sched_barrier(0);
            acc[db] = mma(va[1][db], pf1, acc[db]);
            va[1][db] = lds_frag_t(vn, 16, 32 * db, lane);
            __builtin_amdgcn_sched_barrier(0);
        }
        s = sn;
        if (u + 1 < nT) mask_tail(u + 1);
    };
    for (int u0 = 0; u0 < nT; u0 += DEC_NBUF) {
        body(std::integral_constant<int, 0>{}, u0);
        if (u0 + 1 < nT) body(std::integral_constant<int, 1>{}, u0 + 1);
        if (u0 + 2 < nT) body(std::integral_constant<int, 2>{}, u0 + 2);
        if (u0 + 3 < nT) body(std::integral_constant<int, 3>{}, u0 + 3);
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

// One step of the own-KV role: 32 key rows (the last ones of a run repeated past its end and
// masked) from the wavefront's private 16 KB LDS slot against the G query rows of one request,
// which occupy columns 0..G-1 of one MFMA block.
struct OwnState {
    f32x16 acc[4];
    float m_run, l_run;
};
__device__ __forceinline__ void own_reset(OwnState& st) {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.acc[db][r] = 0.f;
    st.m_run = NEG_BIG;
    st.l_run = 0.f;
}
// nkeys: valid keys of the step (1..32)
__device__ __forceinline__ void own_step(OwnState& st, const bf16x8 (&ka)[8], const bf16x8 (&va)[2][4],
                                         const bf16x8 (&qf)[8], int nkeys, float c, int lg) {
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int t8 = 0; t8 < 8; ++t8) s = mma(ka[t8], qf[t8], s);
    if (nkeys < DEC_SUB) {
        const int thr = nkeys - 1 - 4 * lg;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (8 * (r >> 2) + (r & 3) > thr) s[r] = NEG_BIG;
    }
    float tm = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) tm = fmaxf(tm, s[r]);
    tm = partner_max(tm) * c;
    // the running maximum moves only when exceeded by more than RESCALE_GAP (then O and l are
    // rescaled; rare after a run's first step)
    const float m_new = tm > st.m_run + RESCALE_GAP ? tm : st.m_run;
    if (__any(m_new != st.m_run)) {
        const float alpha = fast_exp2(st.m_run - m_new);
        st.l_run *= alpha;
        st.m_run = m_new;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.acc[db][r] *= alpha;
    }
    float rs = 0.f;
    f32x16 p;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        p[r] = fast_exp2(fmaf(s[r], c, -st.m_run));
        rs += p[r];
    }
    st.l_run += rs;
    const bf16x8 pf0 = pack_frag(p, 0), pf1 = pack_frag(p, 8);
#pragma unroll
    for (int db = 0; db < 4; ++db) {
        st.acc[db] = mma(va[0][db], pf0, st.acc[db]);
        st.acc[db] = mma(va[1][db], pf1, st.acc[db]);
    }
}
// normalised partial O and natural-log lse of the G rows (lanes lc < G) into partial slot `slot`
__device__ __forceinline__ void own_store(const OwnState& st, float* __restrict__ part_o, float* __restrict__ part_l,
                                          size_t slot_row0, int G, int lc, int lg) {
    const float l_tot = st.l_run + partner(st.l_run);
    const float inv = 1.f / l_tot;
    if (lc < G) {
        const size_t slot = slot_row0 + lc;
        float* op = part_o + slot * HD;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                typedef float f32x4 __attribute__((ext_vector_type(4)));
                f32x4 w = {st.acc[db][4 * r4] * inv, st.acc[db][4 * r4 + 1] * inv, st.acc[db][4 * r4 + 2] * inv,
                           st.acc[db][4 * r4 + 3] * inv};
                *reinterpret_cast<f32x4*>(op + 32 * db + 8 * r4 + 4 * lg) = w;
            }
        if (lg == 0) part_l[slot] = (st.m_run + fast_log2(l_tot)) * CART_LN2;
    }
}
// 32 rows x 256 B from row `row0` of a [rows][pitch] tensor (rows past `lim` repeat row lim) into
// the wavefront's slot: 8 direct-to-LDS loads of 4 rows each, per tensor
__device__ __forceinline__ void own_issue(const char* k_row0, const char* v_row0, uint32_t pitch, int lim, char* kt,
                                          char* vt, int lane) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = 4 * i + (lane >> 4);
        const uint32_t off = static_cast<uint32_t>(min(r, lim)) * pitch + (((lane & 15) ^ swz(r)) << 4);
        dma16(k_row0, off, lds_addr(kt) + 4 * i * ROW_B);
        dma16(v_row0, off, lds_addr(vt) + 4 * i * ROW_B);
    }
}
__device__ __forceinline__ void own_frags(const char* kt, const char* vt, bf16x8 (&ka)[8], bf16x8 (&va)[2][4], int lane) {
    const int lg = lane >> 5, lc = lane & 31;
#pragma unroll
    for (int t8 = 0; t8 < 8; ++t8) ka[t8] = lds_frag_n(kt, lc, 16 * t8 + 8 * lg);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int db = 0; db < 4; ++db) va[ks][db] = lds_frag_t(vt, 16 * ks, 32 * db, lane);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}
__device__ __forceinline__ void own_load_q(const bf16_t* __restrict__ q, int b, int Hq, int hk, int G, int lc, int lg,
                                           bf16x8 (&qf)[8]) {
    const bf16_t* qp = q + (static_cast<size_t>(b) * Hq + hk * G + min(lc, G - 1)) * HD + 8 * lg;
#pragma unroll
    for (int t = 0; t < 8; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(qp + 16 * t);
}

// Own-KV role.  The own caches of all requests are one packed tensor [T][Hkv][128], so the work
// is cut evenly along T whatever the requests' lengths: wavefront (range r, KV head hk) streams
// token rows [r*share, (r+1)*share) of head hk, 32 rows per step, without a pause where one
// request ends and the next begins -- the next step's rows are requested before the current step
// is computed, and the next request's query rows are fetched while the current request runs.
// A step never spans two requests (its tail is masked), and every (request, range) pair leaves
// one partial: request b's slot j is range cu[b]/share + j.  Equal bytes per wavefront, all
// wavefronts resident from the start: nothing depends on the order or the pace at which the
// hardware hands out workgroups.  (One workgroup per four (request, head, chunk) items, left
// to the dispatcher, measured 20 us slower on the serving shape: by the middle of the kernel 50
// to 90 CUs sat empty with hundreds of workgroups still to start.)
__device__ __forceinline__ void decode_own_stream(char* sm, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                  const bf16_t* __restrict__ v, const int32_t* __restrict__ cu,
                                                  float* __restrict__ part_o, float* __restrict__ part_l, int B, int Hq,
                                                  int Hkv, float c, int slot0, int n_oc, int share, int wid) {
    const int G = Hq / Hkv;
    const int lane = threadIdx.x & 63, lg = lane >> 5, lc = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = wid / Hkv, hk = wid - r * Hkv;
    const int T = cu[B];
    const long t_lo_l = static_cast<long>(r) * share;
    if (t_lo_l >= T) return;
    const int t_lo = static_cast<int>(t_lo_l);
    const int t_hi = min(t_lo + share, T);
    // the request the range starts in: cu[b] <= t_lo < cu[b+1]
    int cnt = 0;
    for (int i = lane + 1; i <= B; i += 64) cnt += cu[i] <= t_lo ? 1 : 0;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, CART_WAVE);
    int b = __builtin_amdgcn_readfirstlane(cnt);
    if (b >= B) return;                       // (cu not increasing: nothing sensible to do)
    int req_lo = cu[b], req_hi = cu[b + 1];
    int run_end = min(req_hi, t_hi);          // rows [t, run_end) belong to request b
    int next_hi = b + 2 <= B ? cu[b + 2] : T; // end of request b+1
    const uint32_t pitch = static_cast<uint32_t>(Hkv) * ROW_B;
    const char* k_h = reinterpret_cast<const char*>(k) + static_cast<size_t>(hk) * ROW_B;
    const char* v_h = reinterpret_cast<const char*>(v) + static_cast<size_t>(hk) * ROW_B;
    char* kt = sm + (2 * wv) * DEC_SUB_B;
    char* vt = kt + DEC_SUB_B;
    bf16x8 qf[8], qn[8];
    own_load_q(q, b, Hq, hk, G, lc, lg, qf);
    own_load_q(q, min(b + 1, B - 1), Hq, hk, G, lc, lg, qn);
    OwnState st;
    own_reset(st);
    int t = t_lo;
    own_issue(k_h + static_cast<size_t>(t) * pitch, v_h + static_cast<size_t>(t) * pitch, pitch, run_end - 1 - t, kt, vt,
              lane);
    for (;;) {
        const int nkeys = min(DEC_SUB, run_end - t);
        const bool run_last = t + DEC_SUB >= run_end;
        const int t_next = run_last ? run_end : t + DEC_SUB;
        const bool more = t_next < t_hi;
        const int next_end = run_last ? min(next_hi, t_hi) : run_end;
        bf16x8 ka[8], va[2][4];
        dma_wait();                      // this step's rows have landed
        own_frags(kt, vt, ka, va, lane); // into registers; the slot then takes the next step's rows
        if (more)
            own_issue(k_h + static_cast<size_t>(t_next) * pitch, v_h + static_cast<size_t>(t_next) * pitch, pitch,
                      next_end - 1 - t_next, kt, vt, lane);
        own_step(st, ka, va, qf, nkeys, c, lg);
        if (run_last) {
            const int j = r - req_lo / share;
            if (j < n_oc)      // (always, unless a request is longer than the max_own_len the caller stated)
                own_store(st, part_o, part_l, (static_cast<size_t>(slot0 + j) * B + b) * Hq + hk * G, G, lc, lg);
            if (!more) break;
            ++b;
            req_lo = req_hi;
            req_hi = next_hi;
            run_end = next_end;
            next_hi = b + 2 <= B ? cu[b + 2] : T;
#pragma unroll
            for (int i = 0; i < 8; ++i) qf[i] = qn[i];
            own_load_q(q, min(b + 1, B - 1), Hq, hk, G, lc, lg, qn);
            own_reset(st);
        }
        t = t_next;
    }
}

// One chunk of a request's private cartridge pool[cart_id[b]] ([Hkv,pool_p,128]; none when
// cart_id is null or negative), streamed like own rows: item = (request b, chunk cc, KV head hk).
__device__ __forceinline__ void decode_pool_item(char* sm, const bf16_t* __restrict__ q,
                                                 const bf16_t* __restrict__ pool_k, const bf16_t* __restrict__ pool_v,
                                                 const int32_t* __restrict__ cart_id, int pool_p,
                                                 float* __restrict__ part_o, float* __restrict__ part_l, int B, int Hq,
                                                 int Hkv, float c, int chunk, int n_cc, int n_ps, long item) {
    const int G = Hq / Hkv;
    const int lane = threadIdx.x & 63, lg = lane >> 5, lc = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int hk = item % Hkv; item /= Hkv;
    const int cc = item % n_cc;
    const int b = static_cast<int>(item / n_cc);
    const int cid = cart_id ? cart_id[b] : -1;
    if (cid < 0) return;
    const int k0 = cc * chunk;
    if (k0 >= pool_p) return;
    const int nk = min(chunk, pool_p - k0);
    const size_t row0 = (static_cast<size_t>(cid) * Hkv + hk) * pool_p + k0;
    const char* k_b = reinterpret_cast<const char*>(pool_k) + row0 * ROW_B;
    const char* v_b = reinterpret_cast<const char*>(pool_v) + row0 * ROW_B;
    char* kt = sm + (2 * wv) * DEC_SUB_B;
    char* vt = kt + DEC_SUB_B;
    bf16x8 qf[8];
    own_load_q(q, b, Hq, hk, G, lc, lg, qf);
    OwnState st;
    own_reset(st);
    own_issue(k_b, v_b, ROW_B, nk - 1, kt, vt, lane);
    for (int j0 = 0; j0 < nk; j0 += DEC_SUB) {
        bf16x8 ka[8], va[2][4];
        dma_wait();
        own_frags(kt, vt, ka, va, lane);
        if (j0 + DEC_SUB < nk)
            own_issue(k_b + static_cast<size_t>(j0 + DEC_SUB) * ROW_B, v_b + static_cast<size_t>(j0 + DEC_SUB) * ROW_B, ROW_B,
                      nk - 1 - j0 - DEC_SUB, kt, vt, lane);
        own_step(st, ka, va, qf, min(DEC_SUB, nk - j0), c, lg);
    }
    own_store(st, part_o, part_l, (static_cast<size_t>(n_ps + cc) * B + b) * Hq + hk * G, G, lc, lg);
}

// Both roles in one launch, two workgroups per CU: prefix workgroups (matrix-core and LDS work
// on data that sits in L2) and own-KV workgroups (HBM streaming) alternate in the grid while
// both kinds remain, so that the two run side by side instead of one after the other.  The
// launch holds no more workgroups than the chip keeps resident.
__global__ __launch_bounds__(256, 2) void decode_fused_kernel(
    const bf16_t* __restrict__ q, const PrefixTable tab, const bf16_t* __restrict__ k,
    const bf16_t* __restrict__ v, const int32_t* __restrict__ cu, const bf16_t* __restrict__ pool_k,
    const bf16_t* __restrict__ pool_v, const int32_t* __restrict__ cart_id, int pool_p,
    float* __restrict__ part_o, float* __restrict__ part_l, int B, int Hq, int Hkv, float c, int n_rb, int chunk,
    int n_cc, int n_oc, int share, int n_ps, int n_pre_wg, int n_own_wg) {
    constexpr int pre_b = 2 * DEC_NBUF * DEC_TILE_B, own_b = 4 * 2 * DEC_SUB_B;   // the two roles share one LDS block
    __shared__ __attribute__((aligned(16))) char sm[pre_b > own_b ? pre_b : own_b];
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
    if (pre) {
        decode_prefix_role(sm, q, tab, part_o, part_l, B, Hq, Hkv, c, n_rb, idx);
        return;
    }
    // every wavefront on its own from here on: no barrier in this role
    const int wid = __builtin_amdgcn_readfirstlane(idx * 4 + static_cast<int>(threadIdx.x >> 6));
    decode_own_stream(sm, q, k, v, cu, part_o, part_l, B, Hq, Hkv, c, n_ps + n_cc, n_oc, share, wid);
    if (n_cc > 0) {
        const long n_items = static_cast<long>(B) * n_cc * Hkv;
        for (long item = wid; item < n_items; item += 4L * n_own_wg)
            decode_pool_item(sm, q, pool_k, pool_v, cart_id, pool_p, part_o, part_l, B, Hq, Hkv, c, chunk, n_cc, n_ps,
                             item);
    }
}

// o[b,h,:] = sum_i w_i part_o[i] / sum_i w_i, w_i = exp(lse_i - max lse), over the partial slots
// that exist for the request: the n_ps prefix parts, the chunks of its private cartridge (when it
// has one), one per range of `share` token rows its own rows reach into.  One wavefront per
// (b, h), the slots in groups of 64: lane i holds the lse and the weight of the group's slot i,
// then every lane accumulates its two head elements over the group's slots with the loads of
// eight slots in flight.
__global__ __launch_bounds__(256) void decode_merge_kernel(const float* __restrict__ part_o,
                                                           const float* __restrict__ part_l,
                                                           const int32_t* __restrict__ cu,
                                                           const int32_t* __restrict__ cart_id, int pool_p,
                                                           bf16_t* __restrict__ o,
                                                           float* __restrict__ lse, int B, int Hq,
                                                           int n_ps, int n_cc, int n_oc, int chunk, int share) {
    const int lane = threadIdx.x & 63;
    const long row = static_cast<long>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (row >= static_cast<long>(B) * Hq) return;
    const int b = row / Hq;
    const int priv = (n_cc > 0 && cart_id && cart_id[b] >= 0) ? (pool_p + chunk - 1) / chunk : 0;
    const int own = min(n_oc, (cu[b + 1] - 1) / share - cu[b] / share + 1);
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
    const DecodePlan p = make_plan(d.B, d.Hq, d.Hkv, d.max_own_len, d.total_own_tokens, &d.P, d.P > 0 ? 1 : 0, 0);
    return p.part_o_bytes + p.part_l_bytes;
}

bool decode_composed_supported(const cart_decode_composed_desc& d) {
    return d.dtype == CART_BF16 && d.D == 128 && d.Hq / d.Hkv <= 32;
}

static DecodePlan composed_plan(const cart_decode_composed_desc& d, const cart_segment* shared) {
    int seg_p[DEC_MAX_SEG];
    for (int s = 0; s < d.n_shared; ++s) seg_p[s] = shared[s].p;
    return make_plan(d.B, d.Hq, d.Hkv, d.max_own_len, d.total_own_tokens, seg_p, d.n_shared,
                     d.n_pool > 0 ? d.pool_p : 0);
}

size_t decode_composed_workspace(const cart_decode_composed_desc& d, const cart_segment* shared) {
    const DecodePlan p = composed_plan(d, shared);
    return p.part_o_bytes + p.part_l_bytes;
}

// prefix parts + private-cartridge chunks + own ranges (one launch), then the merge
static int run_decode(const DecodePlan& p, int B, int Hq, int Hkv, float scale, const void* q, const void* pool_k,
                      const void* pool_v, const int32_t* cart_id, int pool_p, const void* k, const void* v,
                      const int32_t* cu, void* o, float* lse, void* ws, hipStream_t st) {
    float* part_o = static_cast<float*>(ws);
    float* part_l = reinterpret_cast<float*>(static_cast<char*>(ws) + p.part_o_bytes);
    const float c = scale * CART_LOG2E;
    const bf16_t *Q = static_cast<const bf16_t*>(q), *K = static_cast<const bf16_t*>(k), *V = static_cast<const bf16_t*>(v),
                 *PK = static_cast<const bf16_t*>(pool_k), *PV = static_cast<const bf16_t*>(pool_v);
    trace_begin(st);   // kernel order: prefix + own (one launch), merge
    const int n_pre_wg = p.n_ps > 0 ? p.tab.blk0[p.tab.n_seg] : 0;
    hipLaunchKernelGGL(decode_fused_kernel, dim3(static_cast<unsigned>(n_pre_wg + p.n_own_wg)), dim3(256), 0, st, Q,
                       p.tab, K, V, cu, PK, PV, cart_id, pool_p, part_o, part_l, B, Hq, Hkv, c, p.n_rb, p.chunk, p.n_cc,
                       p.n_oc, p.share, p.n_ps, n_pre_wg, p.n_own_wg);
    trace_mark(st);
    const long rows = static_cast<long>(B) * Hq;
    hipLaunchKernelGGL(decode_merge_kernel, dim3(static_cast<unsigned>((rows + 3) / 4)), dim3(256), 0, st, part_o,
                       part_l, cu, cart_id, pool_p, static_cast<bf16_t*>(o), lse, B, Hq, p.n_ps, p.n_cc, p.n_oc,
                       p.chunk, p.share);
    trace_mark(st);
    return static_cast<int>(hipGetLastError());
}

int launch_decode_mfma(const cart_decode_desc& d, float scale, const void* q, const void* zk,
                       const void* zv, const void* k, const void* v, const int32_t* cu, void* o,
                       float* lse, void* ws, hipStream_t st) {
    DecodePlan p = make_plan(d.B, d.Hq, d.Hkv, d.max_own_len, d.total_own_tokens, &d.P, d.P > 0 ? 1 : 0, 0);
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
