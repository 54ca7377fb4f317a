// Serve-time decode over a shared cartridge (Sec. 3.3; decode step of Sec. 2.3) on the matrix
// cores, bf16, head_dim 128.  One query token per request; keys = [prefix Z ; the request's own
// KV], all visible.
//
// The cartridge is shared by every request, so its part is a real GEMM: the B*G query rows
// that read one KV head (G = Hq/Hkv) are stacked and run against the prefix exactly like the
// training forward kernel, split along the prefix to fill the chip (decode_prefix_kernel).
// The ragged own-KV part is bandwidth-bound: one wavefront per (request, KV head, chunk of
// keys) streams its chunk through a private LDS slot with the G query rows padded into one
// 32-column MFMA block (decode_own_kernel).  Every split writes a normalised partial (O, lse);
// decode_merge_kernel combines them by their log-sum-exps.
#include "attn_mfma.h"

namespace cart {
using namespace mfma;

constexpr int DEC_BM = 256;            // stacked query rows per prefix workgroup
constexpr int DEC_BN = 64;             // prefix keys per LDS tile
constexpr int DEC_NBUF = 3;
constexpr int DEC_TILE_B = DEC_BN * ROW_B;
constexpr int DEC_SUB = 32;            // own keys per wavefront step
constexpr int DEC_SUB_B = DEC_SUB * ROW_B;

struct DecodePlan {
    int G, n_rb, tiles_per_split, n_ps;   // prefix: row blocks, tiles per split, splits
    int chunk, n_oc;                      // own: keys per chunk, chunks per request (worst case)
    size_t part_o_bytes, part_l_bytes;
};

static DecodePlan make_plan(const cart_decode_desc& d) {
    DecodePlan p;
    p.G = d.Hq / d.Hkv;
    const int rows = d.B * p.G;
    p.n_rb = (rows + DEC_BM - 1) / DEC_BM;
    const int nPt = (d.P + DEC_BN - 1) / DEC_BN;
    if (nPt == 0) {
        p.tiles_per_split = 0;
        p.n_ps = 0;
    } else {
        int want = (256 + d.Hkv * p.n_rb - 1) / (d.Hkv * p.n_rb);   // splits to reach ~256 workgroups
        want = want < 1 ? 1 : (want > nPt ? nPt : want);
        p.tiles_per_split = (nPt + want - 1) / want;
        p.n_ps = (nPt + p.tiles_per_split - 1) / p.tiles_per_split;
    }
    p.chunk = d.max_own_len > 4096 ? 1024 : 256;
    p.n_oc = (d.max_own_len + p.chunk - 1) / p.chunk;
    const size_t slots = static_cast<size_t>(p.n_ps + p.n_oc) * d.B * d.Hq;
    p.part_o_bytes = (slots * HD * sizeof(float) + 255) & ~static_cast<size_t>(255);
    p.part_l_bytes = (slots * sizeof(float) + 255) & ~static_cast<size_t>(255);
    return p;
}

struct DecSmem {
    char k[DEC_NBUF][DEC_TILE_B];
    char v[DEC_NBUF][DEC_TILE_B];
};

// acc *= alpha in place in an accumulation register (see the forward kernel)
__device__ __forceinline__ void dec_acc_scale(float& x, float alpha) {
    float tmp;
    asm volatile(
        "s_nop 15\n\tv_accvgpr_read_b32 %1, %0\n\ts_nop 1\n\tv_mul_f32 %1, %1, %2\n\ts_nop 1\n\t"
        "v_accvgpr_write_b32 %0, %1\n\ts_nop 3"
        : "+a"(x), "=&v"(tmp)
        : "v"(alpha));
}

// part_o [split][B][Hq][128] fp32 (normalised), part_l [split][B][Hq] (natural-log lse)
__global__ __launch_bounds__(256, 1) void decode_prefix_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ zk, const bf16_t* __restrict__ zv,
    float* __restrict__ part_o, float* __restrict__ part_l, int B, int Hq, int Hkv, int P, float c,
    int n_rb, int tiles_per_split) {
    __shared__ DecSmem sm;
    const int G = Hq / Hkv;
    int id = blockIdx.x;
    const int hk = id % Hkv; id /= Hkv;
    const int rb = id % n_rb;
    const int sp = id / n_rb;
    const int lane = threadIdx.x & 63, lg = lane >> 5, lc = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rows = B * G;
    const int wrow0 = rb * DEC_BM + 64 * wv;

    bf16x8 qf[2][8];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int rho = min(wrow0 + 32 * cb + lc, rows - 1);
        const bf16_t* qp = q + (static_cast<size_t>(rho / G) * Hq + hk * G + rho % G) * HD + 8 * lg;
#pragma unroll
        for (int t = 0; t < 8; ++t) qf[cb][t] = *reinterpret_cast<const bf16x8*>(qp + 16 * t);
    }
    const int nPt = (P + DEC_BN - 1) / DEC_BN;
    const int t_lo = sp * tiles_per_split;
    const int nT = min(tiles_per_split, nPt - t_lo);
    const char* zk_b = reinterpret_cast<const char*>(zk) + static_cast<size_t>(hk) * P * ROW_B;
    const char* zv_b = reinterpret_cast<const char*>(zv) + static_cast<size_t>(hk) * P * ROW_B;
    auto issue = [&](int t, int buf) __attribute__((always_inline)) {
        const int j0 = (t_lo + t) * DEC_BN;
        tile_load_async<DEC_BN>(sm.k[buf], zk_b, j0, P - 1, ROW_B);
        tile_load_async<DEC_BN>(sm.v[buf], zv_b, j0, P - 1, ROW_B);
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][cb][r] = 0.f;
    float m_run[2] = {NEG_BIG, NEG_BIG}, l_run[2] = {0.f, 0.f};
    f32x16 s[2];
    auto scores = [&](const char* kt, int kr0) __attribute__((always_inline)) {
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[cb][r] = 0.f;
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8) {
            bf16x8 a = lds_frag_n(kt, kr0 + lc, 16 * t8 + 8 * lg);
            s[0] = mma(a, qf[0][t8], s[0]);
            s[1] = mma(a, qf[1][t8], s[1]);
        }
    };
    auto prepare = [&](int t, int hb, bool live) __attribute__((always_inline)) {
        const int j0 = (t_lo + t) * DEC_BN + 32 * hb;
        if (live && j0 + 32 > P) {
            const int thr = P - 1 - j0 - 4 * lg;
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (8 * (r >> 2) + (r & 3) > thr) s[cb][r] = NEG_BIG;
        }
        float m_new[2];
        bool moved = false;
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            float tm = s[cb][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) tm = fmaxf(tm, s[cb][r]);
            tm = partner_max(tm) * c;
            m_new[cb] = (live && tm > m_run[cb] + RESCALE_GAP) ? tm : m_run[cb];
            moved |= m_new[cb] != m_run[cb];
        }
        if (__any(moved)) {
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                const float alpha = fast_exp2(m_run[cb] - m_new[cb]);
                l_run[cb] *= alpha;
                m_run[cb] = m_new[cb];
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float x = acc[db][cb][r];
                        dec_acc_scale(x, alpha);
                        acc[db][cb][r] = x;
                    }
            }
        }
    };

    issue(0, 0);
    dma_wait();
    __syncthreads();
    issue(min(1, nT - 1), 1);
    scores(sm.k[0], 0);
    prepare(0, 0, true);
    const int nU = 2 * nT;
    int buf = 0;
    for (int u = 0; u < nU; ++u) {
        const int hb = u & 1, t = u >> 1;
        const int nbuf = buf + 1 == DEC_NBUF ? 0 : buf + 1;
        const char* vt = sm.v[0] + buf * DEC_TILE_B;
        const char* kt_next = sm.k[0] + (hb ? nbuf : buf) * DEC_TILE_B;
        bf16x8 pf[2][2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            float rs = 0.f;
            f32x16 p;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                p[r] = fast_exp2(fmaf(s[cb][r], c, -m_run[cb]));
                rs += p[r];
            }
            l_run[cb] += rs;
            pf[cb][0] = pack_frag(p, 0);
            pf[cb][1] = pack_frag(p, 8);
        }
        scores(kt_next, hb ? 0 : 32);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                bf16x8 a = lds_frag_t(vt, 32 * hb + 16 * ks, 32 * db, lane);
                acc[db][0] = mma(a, pf[0][ks], acc[db][0]);
                acc[db][1] = mma(a, pf[1][ks], acc[db][1]);
            }
        prepare((u + 1) >> 1, (u + 1) & 1, u + 1 < nU);
        if (!hb) {
            dma_wait();
            __syncthreads();
            issue(min(t + 2, nT - 1), nbuf + 1 == DEC_NBUF ? 0 : nbuf + 1);
        } else {
            buf = nbuf;
        }
    }
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int rho = wrow0 + 32 * cb + lc;
        const float l_tot = l_run[cb] + partner(l_run[cb]);
        const float inv = 1.f / l_tot;
        if (rho < rows) {
            const size_t slot = (static_cast<size_t>(sp) * B + rho / G) * Hq + hk * G + rho % G;
            float* op = part_o + slot * HD;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    typedef float f32x4 __attribute__((ext_vector_type(4)));
                    f32x4 w = {acc[db][cb][4 * r4] * inv, acc[db][cb][4 * r4 + 1] * inv,
                               acc[db][cb][4 * r4 + 2] * inv, acc[db][cb][4 * r4 + 3] * inv};
                    *reinterpret_cast<f32x4*>(op + 32 * db + 8 * r4 + 4 * lg) = w;
                }
            if (lg == 0) part_l[slot] = (m_run[cb] + fast_log2(l_tot)) * CART_LN2;
        }
    }
}

// One wavefront per (request, KV head, chunk of own keys); 32 keys per step through a private
// 16 KB LDS slot.  The G query rows of the group occupy columns 0..G-1 of one MFMA block.
__global__ __launch_bounds__(256, 2) void decode_own_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const int32_t* __restrict__ cu, float* __restrict__ part_o, float* __restrict__ part_l, int B,
    int Hq, int Hkv, float c, int chunk, int n_oc, int n_ps) {
    __shared__ char sm[4][2][DEC_SUB_B];   // [wavefront][K, V]
    const int G = Hq / Hkv;
    const int lane = threadIdx.x & 63, lg = lane >> 5, lc = lane & 31;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    long item = static_cast<long>(blockIdx.x) * 4 + wv;
    const int hk = item % Hkv; item /= Hkv;
    const int cc = item % n_oc;
    const int b = static_cast<int>(item / n_oc);
    if (b >= B) return;
    const int t0 = cu[b], len = cu[b + 1] - t0;
    const int k0 = cc * chunk;
    if (k0 >= len) return;
    const int nk = min(chunk, len - k0);

    bf16x8 qf[8];
    {
        const bf16_t* qp = q + (static_cast<size_t>(b) * Hq + hk * G + min(lc, G - 1)) * HD + 8 * lg;
#pragma unroll
        for (int t = 0; t < 8; ++t) qf[t] = *reinterpret_cast<const bf16x8*>(qp + 16 * t);
    }
    char* kt = sm[wv][0];
    char* vt = sm[wv][1];
    const uint32_t pitch = static_cast<uint32_t>(Hkv) * ROW_B;
    const char* k_b = reinterpret_cast<const char*>(k) + (static_cast<size_t>(t0 + k0) * Hkv + hk) * ROW_B;
    const char* v_b = reinterpret_cast<const char*>(v) + (static_cast<size_t>(t0 + k0) * Hkv + hk) * ROW_B;
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

// o[b,h,:] = sum_i w_i part_o[i] / sum_i w_i, w_i = exp(lse_i - max lse), over the n_ps prefix
// splits and the request's ceil(len/chunk) own chunks.  One wavefront per (b, h): lane i holds
// partial i's lse and weight (n <= 64, else a serial loop), then every lane accumulates its two
// head elements over the partials with the loads of four partials in flight.
__global__ __launch_bounds__(256) void decode_merge_kernel(const float* __restrict__ part_o,
                                                           const float* __restrict__ part_l,
                                                           const int32_t* __restrict__ cu,
                                                           bf16_t* __restrict__ o,
                                                           float* __restrict__ lse, int B, int Hq,
                                                           int n_ps, int chunk) {
    const int lane = threadIdx.x & 63;
    const long row = static_cast<long>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (row >= static_cast<long>(B) * Hq) return;
    const int b = row / Hq;
    const int len = cu[b + 1] - cu[b];
    const int n = n_ps + (len + chunk - 1) / chunk;
    const size_t stride = static_cast<size_t>(B) * Hq;
    float wsum = 0.f, a0 = 0.f, a1 = 0.f, m;
    if (n <= 64) {
        const float li = lane < n ? part_l[lane * stride + row] : -3.0e38f;
        m = wave_max(li);
        const float wi = lane < n ? __expf(li - m) : 0.f;
        wsum = wave_sum(wi);
        int i = 0;
        for (; i + 4 <= n; i += 4) {
            float2 x[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                x[j] = *reinterpret_cast<const float2*>(part_o + ((i + j) * stride + row) * HD + 2 * lane);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float w = __shfl(wi, i + j);
                a0 = fmaf(w, x[j].x, a0);
                a1 = fmaf(w, x[j].y, a1);
            }
        }
        for (; i < n; ++i) {
            const float w = __shfl(wi, i);
            const float2 x = *reinterpret_cast<const float2*>(part_o + (i * stride + row) * HD + 2 * lane);
            a0 = fmaf(w, x.x, a0);
            a1 = fmaf(w, x.y, a1);
        }
    } else {
        m = -3.0e38f;
        for (int i = 0; i < n; ++i) m = fmaxf(m, part_l[i * stride + row]);
        for (int i = 0; i < n; ++i) {
            const float w = __expf(part_l[i * stride + row] - m);
            const float2 x = *reinterpret_cast<const float2*>(part_o + (i * stride + row) * HD + 2 * lane);
            wsum += w;
            a0 = fmaf(w, x.x, a0);
            a1 = fmaf(w, x.y, a1);
        }
    }
    const float inv = 1.f / wsum;
    *reinterpret_cast<uint32_t*>(o + row * HD + 2 * lane) = pack_bf16x2(a0 * inv, a1 * inv);
    if (lane == 0 && lse) lse[row] = m + __logf(wsum);
}

bool decode_mfma_supported(const cart_decode_desc& d) {
    return d.dtype == CART_BF16 && d.D == 128 && d.Hq / d.Hkv <= 32;
}

size_t decode_mfma_workspace(const cart_decode_desc& d) {
    const DecodePlan p = make_plan(d);
    return p.part_o_bytes + p.part_l_bytes;
}

int launch_decode_mfma(const cart_decode_desc& d, float scale, const void* q, const void* zk,
                       const void* zv, const void* k, const void* v, const int32_t* cu, void* o,
                       float* lse, void* ws, hipStream_t st) {
    const DecodePlan p = make_plan(d);
    float* part_o = static_cast<float*>(ws);
    float* part_l = reinterpret_cast<float*>(static_cast<char*>(ws) + p.part_o_bytes);
    const float c = scale * CART_LOG2E;
    // (running the prefix kernel beside the own-KV kernel on a second stream was measured: the
    // event hand-over between the two queues costs more than the overlap gains, 141 vs 131 us)
    trace_begin(st);   // kernel order: prefix, own, merge
    if (p.n_ps > 0) {
        const unsigned grid = static_cast<unsigned>(d.Hkv) * p.n_rb * p.n_ps;
        hipLaunchKernelGGL(decode_prefix_kernel, dim3(grid), dim3(256), 0, st,
                           static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(zk),
                           static_cast<const bf16_t*>(zv), part_o, part_l, d.B, d.Hq, d.Hkv, d.P, c, p.n_rb,
                           p.tiles_per_split);
    }
    trace_mark(st);
    const long items = static_cast<long>(d.B) * d.Hkv * p.n_oc;
    hipLaunchKernelGGL(decode_own_kernel, dim3(static_cast<unsigned>((items + 3) / 4)), dim3(256), 0, st,
                       static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(k),
                       static_cast<const bf16_t*>(v), cu, part_o, part_l, d.B, d.Hq, d.Hkv, c, p.chunk, p.n_oc,
                       p.n_ps);
    trace_mark(st);
    const long rows = static_cast<long>(d.B) * d.Hq;
    hipLaunchKernelGGL(decode_merge_kernel, dim3(static_cast<unsigned>((rows + 3) / 4)), dim3(256), 0, st, part_o,
                       part_l, cu, static_cast<bf16_t*>(o), lse, d.B, d.Hq, p.n_ps, p.chunk);
    trace_mark(st);
    return static_cast<int>(hipGetLastError());
}

}  // namespace cart
