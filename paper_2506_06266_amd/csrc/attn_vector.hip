// fp32 vector-ALU kernels for cartridge attention (Eq. 1 over the cache of Sec. 3.2), its
// gradient, and decode (Sec. 3.3).  One 64-lane wavefront per output row; lane l owns head
// elements l, l+64, ...  They serve fp32 problems and any head_dim <= 256, and are the
// correctness baseline the MFMA kernels are compared with; no atomics, fixed summation order.
#include "cart_common.h"

namespace cart {

constexpr int VEC_MAXE = 4;          // head_dim <= 256
constexpr int VEC_WAVES = 4;         // wavefronts per workgroup

template <typename T, int E>
__device__ __forceinline__ void load_row(const T* p, int D, int lane, float (&r)[E]) {
#pragma unroll
    for (int e = 0; e < E; ++e) {
        int d = lane + 64 * e;
        r[e] = d < D ? elem<T>::load(p + d) : 0.f;
    }
}
template <int E>
__device__ __forceinline__ float dot_rows(const float (&a)[E], const float (&b)[E]) {
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) s = fmaf(a[e], b[e], s);
    return wave_sum(s);
}

// key / value row j of the concatenated cache [prefix ; own] for (sequence b, KV head hk)
template <typename T>
__device__ __forceinline__ const T* cache_row(const T* z, const T* own, int j, int P, int S,
                                              int Hkv, int D, int b, int hk) {
    return j < P ? z + (static_cast<size_t>(hk) * P + j) * D
                 : own + ((static_cast<size_t>(b) * S + (j - P)) * Hkv + hk) * D;
}

template <typename T, int E>
__global__ __launch_bounds__(64 * VEC_WAVES) void attn_fwd_vector(
    const T* q, const T* k, const T* v, const T* zk, const T* zv, T* o, float* lse, int B, int S,
    int Hq, int Hkv, int D, int P, float scale) {
    const int lane = threadIdx.x & 63;
    const long row = static_cast<long>(blockIdx.x) * VEC_WAVES + (threadIdx.x >> 6);
    if (row >= static_cast<long>(B) * S * Hq) return;
    const int h = row % Hq, i = (row / Hq) % S, b = row / (static_cast<long>(Hq) * S);
    const int hk = h / (Hq / Hkv);
    float qr[E], acc[E];
    load_row<T, E>(q + row * D, D, lane, qr);
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.f;
    const float c = scale * CART_LOG2E;
    float m = -3.0e38f, l = 0.f;
    const int nk = P + i + 1;
    for (int j = 0; j < nk; ++j) {
        float kr[E], vr[E];
        load_row<T, E>(cache_row(zk, k, j, P, S, Hkv, D, b, hk), D, lane, kr);
        load_row<T, E>(cache_row(zv, v, j, P, S, Hkv, D, b, hk), D, lane, vr);
        float s = dot_rows<E>(qr, kr) * c;
        float nm = fmaxf(m, s);
        float corr = fast_exp2(m - nm), pj = fast_exp2(s - nm);
        l = l * corr + pj;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = acc[e] * corr + pj * vr[e];
        m = nm;
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        int d = lane + 64 * e;
        if (d < D) elem<T>::store(o + row * D + d, acc[e] * inv);
    }
    if (lane == 0) lse[(static_cast<size_t>(b) * Hq + h) * S + i] = (m + fast_log2(l)) * CART_LN2;
}

// delta[b,h,i] = dO_i . O_i
template <typename T, int E>
__global__ __launch_bounds__(64 * VEC_WAVES) void attn_delta_vector(const T* o, const T* d_o,
                                                                    float* delta, int B, int S,
                                                                    int Hq, int D) {
    const int lane = threadIdx.x & 63;
    const long row = static_cast<long>(blockIdx.x) * VEC_WAVES + (threadIdx.x >> 6);
    if (row >= static_cast<long>(B) * S * Hq) return;
    const int h = row % Hq, i = (row / Hq) % S, b = row / (static_cast<long>(Hq) * S);
    float a[E], g[E];
    load_row<T, E>(o + row * D, D, lane, a);
    load_row<T, E>(d_o + row * D, D, lane, g);
    float s = dot_rows<E>(a, g);
    if (lane == 0) delta[(static_cast<size_t>(b) * Hq + h) * S + i] = s;
}

template <typename T, int E>
__global__ __launch_bounds__(64 * VEC_WAVES) void attn_bwd_dq_vector(
    const T* q, const T* k, const T* v, const T* zk, const T* zv, const float* lse,
    const float* delta, const T* d_o, T* dq, int B, int S, int Hq, int Hkv, int D, int P,
    float scale) {
    const int lane = threadIdx.x & 63;
    const long row = static_cast<long>(blockIdx.x) * VEC_WAVES + (threadIdx.x >> 6);
    if (row >= static_cast<long>(B) * S * Hq) return;
    const int h = row % Hq, i = (row / Hq) % S, b = row / (static_cast<long>(Hq) * S);
    const int hk = h / (Hq / Hkv);
    float qr[E], gr[E], acc[E];
    load_row<T, E>(q + row * D, D, lane, qr);
    load_row<T, E>(d_o + row * D, D, lane, gr);
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.f;
    const size_t st = (static_cast<size_t>(b) * Hq + h) * S + i;
    const float c = scale * CART_LOG2E, l2 = lse[st] * CART_LOG2E, dl = delta[st];
    const int nk = P + i + 1;
    for (int j = 0; j < nk; ++j) {
        float kr[E], vr[E];
        load_row<T, E>(cache_row(zk, k, j, P, S, Hkv, D, b, hk), D, lane, kr);
        load_row<T, E>(cache_row(zv, v, j, P, S, Hkv, D, b, hk), D, lane, vr);
        float p = fast_exp2(dot_rows<E>(qr, kr) * c - l2);
        float ds = p * (dot_rows<E>(gr, vr) - dl);
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = fmaf(ds, kr[e], acc[e]);
    }
#pragma unroll
    for (int e = 0; e < E; ++e) {
        int d = lane + 64 * e;
        if (d < D) elem<T>::store(dq + row * D + d, acc[e] * scale);
    }
}

// One wavefront per key: rows [0, Hkv*P) are prefix slots (summed over every sequence, every
// query head of the group, every token), the rest are own keys (b, j, hk), summed over the
// group's heads and tokens i >= j.
template <typename T, int E>
__global__ __launch_bounds__(64 * VEC_WAVES) void attn_bwd_dkv_vector(
    const T* q, const T* k, const T* v, const T* zk, const T* zv, const float* lse,
    const float* delta, const T* d_o, T* dk, T* dv, float* dzk, float* dzv, int B, int S, int Hq,
    int Hkv, int D, int P, float scale, int n_frozen, int accumulate) {
    const int lane = threadIdx.x & 63;
    const long key = static_cast<long>(blockIdx.x) * VEC_WAVES + (threadIdx.x >> 6);
    const long n_prefix = static_cast<long>(Hkv) * P;
    if (key >= n_prefix + static_cast<long>(B) * S * Hkv) return;
    const bool prefix = key < n_prefix;
    int hk, b0, b1, i0, slot = 0;
    const T *kp, *vp;
    if (prefix) {
        hk = key / P; slot = key % P; b0 = 0; b1 = B; i0 = 0;
        kp = zk + key * D; vp = zv + key * D;
    } else {
        long r = key - n_prefix;
        hk = r % Hkv; i0 = (r / Hkv) % S; b0 = r / (static_cast<long>(Hkv) * S); b1 = b0 + 1;
        kp = k + r * D; vp = v + r * D;
    }
    const int G = Hq / Hkv;
    float kr[E], vr[E], ak[E], av[E];
    load_row<T, E>(kp, D, lane, kr);
    load_row<T, E>(vp, D, lane, vr);
#pragma unroll
    for (int e = 0; e < E; ++e) { ak[e] = 0.f; av[e] = 0.f; }
    const float c = scale * CART_LOG2E;
    for (int b = b0; b < b1; ++b)
        for (int g = 0; g < G; ++g) {
            const int h = hk * G + g;
            for (int i = i0; i < S; ++i) {
                const size_t row = (static_cast<size_t>(b) * S + i) * Hq + h;
                const size_t st = (static_cast<size_t>(b) * Hq + h) * S + i;
                float qr[E], gr[E];
                load_row<T, E>(q + row * D, D, lane, qr);
                load_row<T, E>(d_o + row * D, D, lane, gr);
                float p = fast_exp2(dot_rows<E>(qr, kr) * c - lse[st] * CART_LOG2E);
                float ds = p * (dot_rows<E>(gr, vr) - delta[st]);
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    av[e] = fmaf(p, gr[e], av[e]);
                    ak[e] = fmaf(ds, qr[e], ak[e]);
                }
            }
        }
#pragma unroll
    for (int e = 0; e < E; ++e) {
        int d = lane + 64 * e;
        if (d >= D) continue;
        if (prefix) {
            const bool frozen = slot < n_frozen;
            float gk = frozen ? 0.f : ak[e] * scale, gv = frozen ? 0.f : av[e];
            if (accumulate) { gk += dzk[key * D + d]; gv += dzv[key * D + d]; }
            dzk[key * D + d] = gk;
            dzv[key * D + d] = gv;
        } else {
            long r = key - n_prefix;
            elem<T>::store(dk + r * D + d, ak[e] * scale);
            elem<T>::store(dv + r * D + d, av[e]);
        }
    }
}

template <typename T, int E>
__global__ __launch_bounds__(64 * VEC_WAVES) void decode_vector(
    const T* q, const T* zk, const T* zv, const T* k, const T* v, const int32_t* cu, T* o,
    float* lse, int B, int Hq, int Hkv, int D, int P, float scale) {
    const int lane = threadIdx.x & 63;
    const long row = static_cast<long>(blockIdx.x) * VEC_WAVES + (threadIdx.x >> 6);
    if (row >= static_cast<long>(B) * Hq) return;
    const int h = row % Hq, b = row / Hq;
    const int hk = h / (Hq / Hkv);
    const int t0 = cu[b], len = cu[b + 1] - t0;
    float qr[E], acc[E];
    load_row<T, E>(q + row * D, D, lane, qr);
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.f;
    const float c = scale * CART_LOG2E;
    float m = -3.0e38f, l = 0.f;
    for (int j = 0; j < P + len; ++j) {
        const size_t off = j < P ? (static_cast<size_t>(hk) * P + j) * D
                                 : (static_cast<size_t>(t0 + j - P) * Hkv + hk) * D;
        float kr[E], vr[E];
        load_row<T, E>((j < P ? zk : k) + off, D, lane, kr);
        load_row<T, E>((j < P ? zv : v) + off, D, lane, vr);
        float s = dot_rows<E>(qr, kr) * c;
        float nm = fmaxf(m, s);
        float corr = fast_exp2(m - nm), pj = fast_exp2(s - nm);
        l = l * corr + pj;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = acc[e] * corr + pj * vr[e];
        m = nm;
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        int d = lane + 64 * e;
        if (d < D) elem<T>::store(o + row * D + d, acc[e] * inv);
    }
    if (lane == 0 && lse) lse[row] = (m + fast_log2(l)) * CART_LN2;
}

static inline unsigned blocks_for(long rows) { return static_cast<unsigned>((rows + VEC_WAVES - 1) / VEC_WAVES); }

#define CART_DISPATCH_E(D, BODY)                      \
    do {                                              \
        if ((D) <= 64) { constexpr int E = 1; BODY; } \
        else if ((D) <= 128) { constexpr int E = 2; BODY; } \
        else { constexpr int E = 4; BODY; }           \
    } while (0)

template <typename T>
static void fwd_t(const cart_attn_desc& d, float scale, const void* q, const void* k, const void* v,
                  const void* zk, const void* zv, void* o, float* lse, hipStream_t st) {
    const long rows = static_cast<long>(d.B) * d.S * d.Hq;
    CART_DISPATCH_E(d.D, hipLaunchKernelGGL((attn_fwd_vector<T, E>), dim3(blocks_for(rows)),
        dim3(64 * VEC_WAVES), 0, st, (const T*)q, (const T*)k, (const T*)v, (const T*)zk,
        (const T*)zv, (T*)o, lse, d.B, d.S, d.Hq, d.Hkv, d.D, d.P, scale));
}

int launch_attn_fwd_vector(const cart_attn_desc& d, float scale, const void* q, const void* k,
                           const void* v, const void* zk, const void* zv, void* o, float* lse,
                           hipStream_t st) {
    trace_begin(st);
    if (d.dtype == CART_F32) fwd_t<float>(d, scale, q, k, v, zk, zv, o, lse, st);
    else fwd_t<bf16_t>(d, scale, q, k, v, zk, zv, o, lse, st);
    trace_mark(st);
    return static_cast<int>(hipGetLastError());
}

template <typename T>
static void bwd_t(const cart_attn_desc& d, float scale, const void* q, const void* k, const void* v,
                  const void* zk, const void* zv, const void* o, const float* lse, const void* d_o,
                  void* dq, void* dk, void* dv, float* dzk, float* dzv, void* ws, hipStream_t st) {
    const long rows = static_cast<long>(d.B) * d.S * d.Hq;
    const long keys = static_cast<long>(d.Hkv) * d.P + static_cast<long>(d.B) * d.S * d.Hkv;
    float* delta = static_cast<float*>(ws);
    trace_begin(st);   // kernel order: delta, dq, dk/dv/dz
    CART_DISPATCH_E(d.D, {
        hipLaunchKernelGGL((attn_delta_vector<T, E>), dim3(blocks_for(rows)), dim3(64 * VEC_WAVES),
                           0, st, (const T*)o, (const T*)d_o, delta, d.B, d.S, d.Hq, d.D);
        trace_mark(st);
        hipLaunchKernelGGL((attn_bwd_dq_vector<T, E>), dim3(blocks_for(rows)), dim3(64 * VEC_WAVES),
                           0, st, (const T*)q, (const T*)k, (const T*)v, (const T*)zk, (const T*)zv,
                           lse, delta, (const T*)d_o, (T*)dq, d.B, d.S, d.Hq, d.Hkv, d.D, d.P, scale);
        trace_mark(st);
        hipLaunchKernelGGL((attn_bwd_dkv_vector<T, E>), dim3(blocks_for(keys)), dim3(64 * VEC_WAVES),
                           0, st, (const T*)q, (const T*)k, (const T*)v, (const T*)zk, (const T*)zv,
                           lse, delta, (const T*)d_o, (T*)dk, (T*)dv, dzk, dzv, d.B, d.S, d.Hq,
                           d.Hkv, d.D, d.P, scale, d.n_frozen, d.dz_accumulate);
        trace_mark(st);
    });
}

int launch_attn_bwd_vector(const cart_attn_desc& d, float scale, const void* q, const void* k,
                           const void* v, const void* zk, const void* zv, const void* o,
                           const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                           float* dzk, float* dzv, void* ws, hipStream_t st) {
    if (d.dtype == CART_F32) bwd_t<float>(d, scale, q, k, v, zk, zv, o, lse, d_o, dq, dk, dv, dzk, dzv, ws, st);
    else bwd_t<bf16_t>(d, scale, q, k, v, zk, zv, o, lse, d_o, dq, dk, dv, dzk, dzv, ws, st);
    return static_cast<int>(hipGetLastError());
}

template <typename T>
static void dec_t(const cart_decode_desc& d, float scale, const void* q, const void* zk,
                  const void* zv, const void* k, const void* v, const int32_t* cu, void* o,
                  float* lse, hipStream_t st) {
    const long rows = static_cast<long>(d.B) * d.Hq;
    CART_DISPATCH_E(d.D, hipLaunchKernelGGL((decode_vector<T, E>), dim3(blocks_for(rows)),
        dim3(64 * VEC_WAVES), 0, st, (const T*)q, (const T*)zk, (const T*)zv, (const T*)k,
        (const T*)v, cu, (T*)o, lse, d.B, d.Hq, d.Hkv, d.D, d.P, scale));
}

int launch_decode_vector(const cart_decode_desc& d, float scale, const void* q, const void* zk,
                         const void* zv, const void* k, const void* v, const int32_t* cu,
                         void* o, float* lse, hipStream_t st) {
    trace_begin(st);
    if (d.dtype == CART_F32) dec_t<float>(d, scale, q, zk, zv, k, v, cu, o, lse, st);
    else dec_t<bf16_t>(d, scale, q, zk, zv, k, v, cu, o, lse, st);
    trace_mark(st);
    return static_cast<int>(hipGetLastError());
}

}  // namespace cart
