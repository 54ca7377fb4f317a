// Cartridge attention forward on the matrix cores (bf16 in, fp32 accumulate, head_dim 128):
// Eq. 1 over the cache of Sec. 3.2, [prefix Z (all visible) ; own keys (causal)].
//
// One 256-thread workgroup = 256 consecutive queries of one (sequence, query head); each of its
// four wavefronts owns 64 of them, kept in registers as MFMA operand fragments.  Keys/values
// stream through LDS in tiles of 64 (prefix tiles first, then own tiles up to the diagonal),
// double-buffered, one barrier per tile.  Per tile a wavefront computes S^T = K Q^T (keys on
// the D rows, its queries on the D columns), does the online softmax per lane (a lane owns one
// query, so the running max / sum are lane scalars), and accumulates O^T += V^T P^T with V read
// through the transposing LDS load.
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

// acc *= alpha for an accumulator element that lives in an accumulation register, in place.
// Written as one asm statement so that the rarely taken rescale path does not make the
// compiler carry the O accumulators in ordinary vector registers around the whole loop.  The
// s_nops cover the matrix-core write -> accumulator read latency.
__device__ __forceinline__ void acc_scale(float& x, float alpha) {
    float tmp;
    asm volatile(
        "s_nop 15\n\tv_accvgpr_read_b32 %1, %0\n\ts_nop 1\n\tv_mul_f32 %1, %1, %2\n\ts_nop 1\n\t"
        "v_accvgpr_write_b32 %0, %1\n\ts_nop 3"
        : "+a"(x), "=&v"(tmp)
        : "v"(alpha));
}

__global__ __launch_bounds__(256, 1) void attn_fwd_mfma_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ zk, const bf16_t* __restrict__ zv, bf16_t* __restrict__ o,
    float* __restrict__ lse, int B, int S, int Hq, int Hkv, int P, float c /* scale*log2(e) */) {
    __shared__ FwdSmem sm;
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

    // this wavefront's 64 queries as B-operand fragments: column = query, k = head element
    bf16x8 qf[2][8];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        int qi = wrow0 + 32 * cb + lc;
        qi = qi < S ? qi : S - 1;
        const bf16_t* qp = q + ((static_cast<size_t>(b) * S + qi) * Hq + h) * HD + 8 * lg;
#pragma unroll
        for (int t = 0; t < 8; ++t) qf[cb][t] = *reinterpret_cast<const bf16x8*>(qp + 16 * t);
    }

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
        const size_t pitch = pre ? static_cast<size_t>(ROW_B) : own_pitch;
        const char* kb = pre ? zk_b : k_b;
        const char* vb = pre ? zv_b : v_b;
        tile_load_async<FWD_BN>(sm.k[buf], [&](int r) { return kb + min(j0 + r, last) * pitch; });
        tile_load_async<FWD_BN>(sm.v[buf], [&](int r) { return vb + min(j0 + r, last) * pitch; });
    };

    f32x16 acc[4][2];   // O^T: [head-element block][query block]
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][cb][r] = 0.f;
    float m_run[2] = {NEG_BIG, NEG_BIG}, l_run[2] = {0.f, 0.f};
    f32x16 s[2];        // scores of the sub-tile about to be consumed: 32 keys x 64 queries

    // S^T of 32 keys (tile rows kr0 ..) x this wavefront's queries
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
    // Mask the fresh scores of sub-tile (tile t, half hb), move the running max if some score
    // exceeds it by more than RESCALE_GAP.  live = false (past the last sub-tile) does nothing.
    auto prepare = [&](int t, int hb, bool masked, bool live) __attribute__((always_inline)) {
        if (masked) {
            const bool own = t >= nPt;
            const int j0 = (own ? t - nPt : t) * FWD_BN + 32 * hb;
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                // key j0 + d_row(r, lg) is hidden when it exceeds the lane's last visible key
                const int thr = (own ? wrow0 + 32 * cb + lc : P - 1) - j0 - 4 * lg;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (8 * (r >> 2) + (r & 3) > thr) s[cb][r] = NEG_BIG;
            }
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
                        acc_scale(x, alpha);
                        acc[db][cb][r] = x;
                    }
            }
        }
    };
    // does sub-tile u = 2 t + hb hold a key that some query of this wavefront must not see?
    auto needs_mask = [&](int t, int hb) __attribute__((always_inline)) {
        return t < nPt ? (t * FWD_BN + 32 * hb + 32 > P) : ((t - nPt) * FWD_BN + 32 * hb + 31 > wrow0);
    };

    // Software pipeline over sub-tiles of 32 keys.  At the top of iteration u, s holds the
    // prepared scores of sub-tile u.  The vector ALU turns them into P while the matrix cores
    // compute the scores of sub-tile u+1, then the matrix cores accumulate O^T += V^T P^T.
    // Three LDS buffers; the one barrier per tile comes after a tile's first sub-tile: it
    // publishes tile t+1 (whose scores the next iteration computes ahead) and retires tile t-1's
    // buffer, which then receives tile t+2.
    issue(0, 0);
    __syncthreads();
    issue(min(1, nT - 1), 1);
    scores(sm.k[0], 0);
    prepare(0, 0, needs_mask(0, 0), true);
    const int nU = 2 * nT;
    int buf = 0;                      // LDS buffer of the tile sub-tile u belongs to
    for (int u = 0; u < nU; ++u) {
        const int hb = u & 1, t = u >> 1;
        const int nbuf = buf + 1 == FWD_NBUF ? 0 : buf + 1;
        const char* vt = sm.v[0] + buf * FWD_TILE_B;
        const char* kt_next = sm.k[0] + (hb ? nbuf : buf) * FWD_TILE_B;
        bf16x8 pf[2][2];   // [query block][k-step]: P^T as B-operand fragments
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
        const int tn = (u + 1) >> 1, hn = (u + 1) & 1;
        const bool live = u + 1 < nU;
        prepare(tn, hn, live && needs_mask(tn, hn), live);
        if (!hb) {
            __syncthreads();
            issue(min(t + 2, nT - 1), nbuf + 1 == FWD_NBUF ? 0 : nbuf + 1);
        } else {
            buf = nbuf;
        }
    }

    // normalise and store: lane holds, for its query, head elements 32db + 8(r/4) + 4g + r%4
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int qi = wrow0 + 32 * cb + lc;
        const float l_tot = l_run[cb] + partner(l_run[cb]);
        const float inv = 1.f / l_tot;
        if (qi < S) {
            bf16_t* op = o + ((static_cast<size_t>(b) * S + qi) * Hq + h) * HD;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    u32x2 w = {pack_bf16x2(acc[db][cb][4 * r4] * inv, acc[db][cb][4 * r4 + 1] * inv),
                               pack_bf16x2(acc[db][cb][4 * r4 + 2] * inv, acc[db][cb][4 * r4 + 3] * inv)};
                    *reinterpret_cast<u32x2*>(op + 32 * db + 8 * r4 + 4 * lg) = w;
                }
            if (lg == 0)
                lse[(static_cast<size_t>(b) * Hq + h) * S + qi] = (m_run[cb] + fast_log2(l_tot)) * CART_LN2;
        }
    }
}

bool attn_mfma_supported(const cart_attn_desc& d) {
    return d.dtype == CART_BF16 && d.D == 128;
}
size_t attn_mfma_fwd_workspace(const cart_attn_desc&) { return 0; }

int launch_attn_fwd_mfma(const cart_attn_desc& d, float scale, const void* q, const void* k,
                         const void* v, const void* zk, const void* zv, void* o, float* lse,
                         void*, hipStream_t st) {
    const int nQt = (d.S + FWD_BM - 1) / FWD_BM;
    const long grid = static_cast<long>(nQt) * d.B * d.Hq;
    trace_begin(st);
    hipLaunchKernelGGL(attn_fwd_mfma_kernel, dim3(static_cast<unsigned>(grid)), dim3(256), 0, st,
                       static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(k),
                       static_cast<const bf16_t*>(v), static_cast<const bf16_t*>(zk),
                       static_cast<const bf16_t*>(zv), static_cast<bf16_t*>(o), lse, d.B, d.S, d.Hq,
                       d.Hkv, d.P, scale * CART_LOG2E);
    trace_mark(st);
    return static_cast<int>(hipGetLastError());
}

}  // namespace cart
