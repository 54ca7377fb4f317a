// Context-distillation loss (Eq. 3, Sec. 4.2, over the teacher's recorded top entries of
// App. A.2) fused with its gradient: one streaming pass over the student's logits.  Two
// readings of the truncated teacher (recorded terms only / plus a rest bucket) share the pass:
// they differ in one per-row coefficient and in the k fix-ups; next-token cross-entropy is the
// case of one recorded token of probability 1.
//
// kl_row_resident: one 1024-thread workgroup per position holds the whole bf16 row
// (<= 131072 logits) in registers, so HBM sees each logit read once and each gradient written
// once.  Three sweeps over the registers: max, sum of exponentials, gradient.
// kl_row_stream: any vocabulary size / fp32 logits; reads the row twice.
#include "cart_common.h"

namespace cart {

constexpr int KL_MAXK = 1024;

struct KlTeacher {      // per-row teacher records staged in LDS
    int idx[KL_MAXK];
    float t[KL_MAXK];   // exp(logp), 0 for ignored entries
    float lp[KL_MAXK];
    float x[KL_MAXK];   // student logit at idx (read before anything is overwritten)
};

template <typename T, int THREADS>
__device__ __forceinline__ float kl_stage_teacher(KlTeacher& tc, const T* logits_row,
                                                  const int32_t* idx, const float* logp, int V,
                                                  int K) {
    float m_part = 0.f;
    for (int j = threadIdx.x; j < K; j += THREADS) {
        int id = idx[j];
        float lp = logp ? logp[j] : 0.f;
        bool ok = id >= 0 && id < V;
        float t = ok ? __expf(lp) : 0.f;
        tc.idx[j] = ok ? id : -1;
        tc.t[j] = t;
        tc.lp[j] = ok ? lp : 0.f;
        tc.x[j] = ok ? elem<T>::load(logits_row + id) : 0.f;
        m_part += t;
    }
    return m_part;
}

// KL_n = sum_j t_j (logp_j - x_j + lse) (+ extra, the rest-bucket term), by the first wavefront
__device__ __forceinline__ void kl_row_value(const KlTeacher& tc, int K, float lse, float extra, float* out) {
    if (threadIdx.x < CART_WAVE) {
        float a = 0.f;
        for (int j = threadIdx.x; j < K; j += CART_WAVE) a += tc.t[j] * (tc.lp[j] - tc.x[j] + lse);
        a = wave_sum(a);
        if (threadIdx.x == 0) *out = a + extra;
    }
}

// Rest-bucket mode, once the row's log2-sum-exp is known.  The first wavefront sums the student's
// mass on the recorded tokens, S = sum_j 2^(x_j log2e - lse2), and leaves in LDS the coefficient
// of the off-support gradient, (M - S) / (1 - S), and the row's extra term
// (1 - M)(log(1 - M) - log(1 - S)); the caller synchronises before reading them.  1 - M is
// floored at 0 and 1 - S at 2^-24, below which fp32 cannot resolve them.
__device__ __forceinline__ void kl_rest_terms(const KlTeacher& tc, int K, float lse2, float M, float* out2) {
    if (threadIdx.x < CART_WAVE) {
        float a = 0.f;
        for (int j = threadIdx.x; j < K; j += CART_WAVE)
            if (tc.idx[j] >= 0) a += fast_exp2(fmaf(tc.x[j], CART_LOG2E, -lse2));
        a = wave_sum(a);
        if (threadIdx.x == 0) {
            const float rs = fmaxf(1.f - a, 5.9604645e-8f), rt = fmaxf(1.f - M, 0.f);
            out2[0] = (M - a) / rs;
            out2[1] = rt > 0.f ? rt * (__logf(rt) - __logf(rs)) : 0.f;
        }
    }
}

// max of a float and two raw fp32 bit patterns in one instruction, without the NaN-quieting
// moves the compiler would add around fmaxf for values it cannot prove canonical
__device__ __forceinline__ float max3_raw(float a, uint32_t b, uint32_t c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
// Makes the register-resident row opaque to the optimiser between sweeps; otherwise the
// unpacked fp32 copies of one sweep are kept alive for the next one and spill.
#define KL_FORGET(x)                                                                      \
    _Pragma("unroll") for (int i_ = 0; i_ < NV; ++i_)                                      \
        asm volatile("" : "+v"(x[i_].x), "+v"(x[i_].y), "+v"(x[i_].z), "+v"(x[i_].w))

#ifndef KL_RESIDENT_WGS
#define KL_RESIDENT_WGS 256      // workgroups of the register-resident kernel: one per CU of an MI355X
#endif

template <int NV>
__global__ __launch_bounds__(1024) void kl_row_resident(const bf16_t* logits, const int32_t* idx,
                                                        const float* logp, bf16_t* dlogits,
                                                        float* row_kl, int N, int V, int K, float scale,
                                                        int rest) {
    constexpr int THREADS = 1024, NW = THREADS / CART_WAVE;
    __shared__ KlTeacher tc;
    __shared__ float red_max[NW], red_m[NW], red_sum[NW], rest_terms[2];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int nvec = V >> 3;
    const uint32_t FILL = 0xff7fff7fu;   // two bf16 of the most negative finite value

    // One workgroup fills a CU, so nothing else would cover the latency of a row's load: the
    // workgroup walks rows n, n + gridDim.x, ... and fetches the next row into the registers of
    // the current one as the last sweep releases them.
    int n = blockIdx.x;
    if (n >= N) return;
    u32x4 x[NV];
    {
        const u32x4* src = reinterpret_cast<const u32x4*>(logits + static_cast<size_t>(n) * V);
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            int v = i * THREADS + tid;
            x[i] = u32x4{FILL, FILL, FILL, FILL};
            if (v < nvec) x[i] = __builtin_nontemporal_load(src + v);
        }
    }
    for (;;) {
        const size_t row = static_cast<size_t>(n) * V;
        float m_part = kl_stage_teacher<bf16_t, THREADS>(tc, logits + row, idx + static_cast<size_t>(n) * K,
                                                        logp ? logp + static_cast<size_t>(n) * K : nullptr, V, K);

        // sweep 1: the row maximum; both elements of a packed word widened to fp32 (a word of two
        // -inf logits read whole would be a NaN) and a three-way maximum
        float mx = -3.0e38f;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint32_t w[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) mx = max3_raw(mx, w[e] & 0xffff0000u, w[e] << 16);
        }
        KL_FORGET(x);
        mx = wave_max(mx);
        m_part = wave_sum(m_part);
        if (lane == 0) { red_max[wv] = mx; red_m[wv] = m_part; }
        __syncthreads();
        float M = 0.f;
        mx = red_max[0];
#pragma unroll
        for (int w = 0; w < NW; ++w) { mx = fmaxf(mx, red_max[w]); M += red_m[w]; }

        // sweep 2: sum of exp(x - max), in base 2
        const float c0 = -mx * CART_LOG2E;
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint32_t w[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                s0 += fast_exp2(fmaf(__uint_as_float(w[e] << 16), CART_LOG2E, c0));
                s1 += fast_exp2(fmaf(__uint_as_float(w[e] & 0xffff0000u), CART_LOG2E, c0));
            }
            __builtin_amdgcn_sched_barrier(0);   // keep the sweeps' temporaries from piling up
        }
        KL_FORGET(x);
        float sum = wave_sum(s0 + s1);
        if (lane == 0) red_sum[wv] = sum;
        __syncthreads();
        sum = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += red_sum[w];
        const float lse2 = fast_log2(sum) - c0;          // log2 of the softmax denominator

        // sweep 3: g = c * exp(x - lse) with c = scale * M (rest-bucket mode: the off-support
        // coefficient scale * (M - S) / (1 - S)); |c| rides in the exponent.  Each vector's
        // registers take the same vector of the next row as soon as its gradient is stored.
        float coef = M, extra = 0.f;
        if (rest) {
            kl_rest_terms(tc, K, lse2, M, rest_terms);
            __syncthreads();
            coef = rest_terms[0];
            extra = rest_terms[1];
        }
        const float c = scale * coef;
        const float off = -(lse2 - fast_log2(fabsf(c)));  // c == 0 gives -inf, hence g == 0
        const uint32_t sgn = c < 0.f ? 0x80008000u : 0u;
        u32x4* dst = reinterpret_cast<u32x4*>(dlogits + row);
        const int n_next = n + static_cast<int>(gridDim.x);
        const bool more = n_next < N;
        const u32x4* src_next = reinterpret_cast<const u32x4*>(logits + static_cast<size_t>(more ? n_next : n) * V);
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            int v = i * THREADS + tid;
            const uint32_t w[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
            uint32_t r[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float lo = fast_exp2(fmaf(__uint_as_float(w[e] << 16), CART_LOG2E, off));
                float hi = fast_exp2(fmaf(__uint_as_float(w[e] & 0xffff0000u), CART_LOG2E, off));
                r[e] = pack_bf16x2(lo, hi) ^ sgn;
            }
            if (v < nvec) __builtin_nontemporal_store(u32x4{r[0], r[1], r[2], r[3]}, dst + v);
            x[i] = u32x4{FILL, FILL, FILL, FILL};
            if (more && v < nvec) x[i] = __builtin_nontemporal_load(src_next + v);
            __builtin_amdgcn_sched_barrier(0);
        }
        // recorded tokens: the thread that stored the vector holding idx_j rewrites that element,
        // so the two stores to one address are in program order
        for (int j = 0; j < K; ++j) {
            int id = tc.idx[j];
            if (id >= 0 && ((id >> 3) & (THREADS - 1)) == tid) {
                float s = fast_exp2(fmaf(tc.x[j], CART_LOG2E, -lse2));
                dlogits[row + id] = f32_to_bf16(scale * ((rest ? 1.f : M) * s - tc.t[j]));
            }
        }
        kl_row_value(tc, K, lse2 * CART_LN2, extra, row_kl + n);
        if (!more) break;
        n = n_next;
        __syncthreads();    // the teacher staging area and the reduction arrays are reused
    }
}

template <typename T>
__global__ __launch_bounds__(256) void kl_row_stream(const T* logits, const int32_t* idx,
                                                     const float* logp, T* dlogits, float* row_kl,
                                                     int V, int K, float scale, int rest) {
    constexpr int THREADS = 256, NW = THREADS / CART_WAVE;
    __shared__ KlTeacher tc;
    __shared__ float red_max[NW], red_m[NW], red_sum[NW], rest_terms[2];
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const size_t row = static_cast<size_t>(n) * V;
    const T* src = logits + row;

    float m_part = kl_stage_teacher<T, THREADS>(tc, src, idx + static_cast<size_t>(n) * K,
                                               logp ? logp + static_cast<size_t>(n) * K : nullptr, V, K);
    // pass 1: running (max, sum) per thread in base 2
    float mx = -3.0e38f, sum = 0.f;
    for (int v = tid; v < V; v += THREADS) {
        float y = elem<T>::load(src + v) * CART_LOG2E;
        float nm = fmaxf(mx, y);
        sum = sum * fast_exp2(mx - nm) + fast_exp2(y - nm);
        mx = nm;
    }
    float wmx = wave_max(mx);
    sum = wave_sum(sum * fast_exp2(mx - wmx));
    m_part = wave_sum(m_part);
    if (lane == 0) { red_max[wv] = wmx; red_sum[wv] = sum; red_m[wv] = m_part; }
    __syncthreads();
    float M = 0.f, gmx = red_max[0];
#pragma unroll
    for (int w = 0; w < NW; ++w) { gmx = fmaxf(gmx, red_max[w]); M += red_m[w]; }
    sum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) sum += red_sum[w] * fast_exp2(red_max[w] - gmx);
    const float lse2 = gmx + fast_log2(sum);

    // pass 2: gradient; each thread rewrites the recorded tokens it owns after its own stores
    float coef = M, extra = 0.f;
    if (rest) {
        kl_rest_terms(tc, K, lse2, M, rest_terms);
        __syncthreads();
        coef = rest_terms[0];
        extra = rest_terms[1];
    }
    const float c = scale * coef;
    T* dst = dlogits + row;
    for (int v = tid; v < V; v += THREADS) {
        float y = elem<T>::load(src + v);
        elem<T>::store(dst + v, c * fast_exp2(fmaf(y, CART_LOG2E, -lse2)));
    }
    for (int j = 0; j < K; ++j) {
        int id = tc.idx[j];
        if (id >= 0 && (id & (THREADS - 1)) == tid) {
            float s = fast_exp2(fmaf(tc.x[j], CART_LOG2E, -lse2));
            elem<T>::store(dst + id, scale * ((rest ? 1.f : M) * s - tc.t[j]));
        }
    }
    kl_row_value(tc, K, lse2 * CART_LN2, extra, row_kl + n);
}

// loss = scale * sum_n row_kl[n]: one workgroup, fixed summation order, fp64 accumulation
__global__ __launch_bounds__(1024) void kl_reduce_rows(const float* row_kl, int N, float scale,
                                                       float* loss) {
    __shared__ double red[1024];
    double a = 0.0;
    for (int i = threadIdx.x; i < N; i += 1024) a += static_cast<double>(row_kl[i]);
    red[threadIdx.x] = a;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = static_cast<float>(static_cast<double>(scale) * red[0]);
}

int launch_kl(const cart_kl_desc& d, const void* logits, const int32_t* idx, const float* logp,
              float* loss, void* d_logits, float* row_kl, void* ws, hipStream_t st) {
    float* rows = row_kl ? row_kl : static_cast<float*>(ws);
    const int rest = d.mode == CART_KL_REST ? 1 : 0;
    trace_begin(st);   // kernel order: row kernel, loss reduce
    const bool resident = d.logits_dtype == CART_BF16 && (d.V % 8) == 0 && d.V <= 1024 * 16 * 8;
    if (resident) {
        const bf16_t* x = static_cast<const bf16_t*>(logits);
        bf16_t* g = static_cast<bf16_t*>(d_logits);
        const int nvec = d.V / 8;
        const dim3 grid(static_cast<unsigned>(d.N < KL_RESIDENT_WGS ? d.N : KL_RESIDENT_WGS));
        if (nvec <= 1024 * 4)
            hipLaunchKernelGGL(kl_row_resident<4>, grid, dim3(1024), 0, st, x, idx, logp, g, rows, d.N, d.V, d.K, d.scale, rest);
        else if (nvec <= 1024 * 8)
            hipLaunchKernelGGL(kl_row_resident<8>, grid, dim3(1024), 0, st, x, idx, logp, g, rows, d.N, d.V, d.K, d.scale, rest);
        else
            hipLaunchKernelGGL(kl_row_resident<16>, grid, dim3(1024), 0, st, x, idx, logp, g, rows, d.N, d.V, d.K, d.scale, rest);
    } else if (d.logits_dtype == CART_BF16) {
        hipLaunchKernelGGL(kl_row_stream<bf16_t>, dim3(d.N), dim3(256), 0, st,
                           static_cast<const bf16_t*>(logits), idx, logp,
                           static_cast<bf16_t*>(d_logits), rows, d.V, d.K, d.scale, rest);
    } else {
        hipLaunchKernelGGL(kl_row_stream<float>, dim3(d.N), dim3(256), 0, st,
                           static_cast<const float*>(logits), idx, logp,
                           static_cast<float*>(d_logits), rows, d.V, d.K, d.scale, rest);
    }
    trace_mark(st);
    hipLaunchKernelGGL(kl_reduce_rows, dim3(1), dim3(1024), 0, st, rows, d.N, d.scale, loss);
    trace_mark(st);
    return static_cast<int>(hipGetLastError());
}

}  // namespace cart
