// Teacher records (App. A.2 "Training Objective": the top output probabilities of the teacher are
// collected while it generates): per position, the K most probable tokens and their
// log-probabilities, by descending probability, the lower token index first among equal logits.
//
// One workgroup per position; a single pass over the logits.  topk_row_one_pass (the default for
// bf16 rows, K <= 256) is described at the kernel.
// topk_row_resident: 1024 threads hold the whole bf16 row (<= 131072 logits) in registers.  After
// the log-sum-exp (as in the loss kernel) the K largest are found without sorting the row:
//   1. every thread takes the maximum of its 128 logits; the K-th largest of these 1024 maxima,
//      tau, is found by a bitwise binary search over the 16-bit order-preserving key of a bf16
//      (16 rounds of compare + count by one wavefront: no barriers in between).  K distinct logits are >= tau, so the K-th largest logit
//      of the row is >= tau as well: every winner has key >= tau;
//   2. the logits with key >= tau (K plus a few, ties included) go to a list in LDS;
//   3. each listed logit counts the listed logits that precede it in the order (larger value,
//      or equal value and lower index): that count is its output position.
// A row whose list would not fit (thousands of logits tied at the top) is handled by K rounds of
// "best logit after the previous winner" over the row in memory instead.  topk_row_stream does
// those K rounds for fp32 logits or a vocabulary that is not a multiple of 8.
#include "cart_common.h"

namespace cart {

constexpr int TOPK_MAXK = 1024;
constexpr int TOPK_CAP = 4096;        // list capacity (entries)

// max of a float and two raw fp32 bit patterns in one instruction, without the NaN-quieting
// moves the compiler would add around fmaxf for values it cannot prove canonical
__device__ __forceinline__ float max3_raw(float a, uint32_t b, uint32_t c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// order-preserving 16-bit key of a bf16: larger key <=> larger value
__device__ __forceinline__ uint32_t bf16_key(uint32_t bits) {
    if (bits == 0x8000u) bits = 0u;      // -0 and +0 are one value (ties go by index)
    return (bits & 0x8000u) ? (~bits & 0xffffu) : (bits | 0x8000u);
}
__device__ __forceinline__ float bf16_key_value(uint32_t key) {
    const uint32_t bits = (key & 0x8000u) ? (key & 0x7fffu) : (~key & 0xffffu);
    return __uint_as_float(bits << 16);
}
// order-preserving 32-bit key of an fp32
__device__ __forceinline__ uint32_t f32_key(float x) {
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float f32_key_value(uint32_t key) {
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

// (key, index) -> one 64-bit word whose order is "larger value first, then lower index"
__device__ __forceinline__ uint64_t order_word(uint32_t key, uint32_t idx) {
    return (static_cast<uint64_t>(key) << 32) | (0xffffffffu - idx);
}
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint64_t w = __shfl_xor(v, o, CART_WAVE);
        v = w > v ? w : v;
    }
    return v;
}

// K rounds over a thread's own elements: in each round the workgroup's best order word strictly
// below the previous winner.  next(prev) returns the thread's best word < prev (0 when none).
template <int NW, typename Next>
__device__ __forceinline__ void select_rounds(int K, uint64_t* red, Next next, int32_t* idx_out, float* logp_out,
                                              float lse, bool is_bf16) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    uint64_t prev = ~0ull;
    for (int j = 0; j < K; ++j) {
        uint64_t best = wave_max_u64(next(prev));
        if (lane == 0) red[wv] = best;
        __syncthreads();
        best = red[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) best = red[w] > best ? red[w] : best;
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t key = static_cast<uint32_t>(best >> 32);
            idx_out[j] = static_cast<int32_t>(0xffffffffu - static_cast<uint32_t>(best));
            logp_out[j] = (is_bf16 ? bf16_key_value(key) : f32_key_value(key)) - lse;
        }
        prev = best;
    }
}

// Makes the register-resident row opaque to the optimiser between sweeps; otherwise the
// unpacked copies of one sweep are kept alive for the next one and spill.
#define TOPK_FORGET(x)                                                                    \
    _Pragma("unroll") for (int i_ = 0; i_ < NV; ++i_)                                      \
        asm volatile("" : "+v"(x[i_].x), "+v"(x[i_].y), "+v"(x[i_].z), "+v"(x[i_].w))

template <int NV>
__global__ __launch_bounds__(1024) void topk_row_resident(const bf16_t* logits, int32_t* idx_out,
                                                          float* logp_out, int V, int K) {
    constexpr int THREADS = 1024, NW = THREADS / CART_WAVE;
    __shared__ float red_f[NW];
    __shared__ __align__(16) uint16_t all_kmax[THREADS];
    __shared__ uint64_t red_w[NW];
    __shared__ uint32_t list_key[TOPK_CAP];
    __shared__ uint32_t list_idx[TOPK_CAP];
    __shared__ int list_n;
    __shared__ uint32_t tau_s;
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const u32x4* src = reinterpret_cast<const u32x4*>(logits + static_cast<size_t>(n) * V);
    const int nvec = V >> 3;
    idx_out += static_cast<size_t>(n) * K;
    logp_out += static_cast<size_t>(n) * K;

    u32x4 x[NV];
    // two bf16 of the most negative finite value (as a packed fp32 word it is finite too, which
    // the maximum below relies on); positions past V are kept out of the list by their index
    const uint32_t FILL = 0xff7fff7fu;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int v = i * THREADS + tid;
        x[i] = u32x4{FILL, FILL, FILL, FILL};
        if (v < nvec) x[i] = __builtin_nontemporal_load(src + v);
    }
    if (tid == 0) list_n = 0;

    // The thread's largest logit, then the row maximum: both elements of a packed word widened
    // to fp32 (exact; a word of two -inf read whole would be a NaN) and a three-way maximum.
    float tmax = __uint_as_float(0xff800000u);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const uint32_t w[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) tmax = max3_raw(tmax, w[e] & 0xffff0000u, w[e] << 16);
    }
    TOPK_FORGET(x);
    const uint32_t kmax = bf16_key(__float_as_uint(tmax) >> 16);
    all_kmax[tid] = static_cast<uint16_t>(kmax);
    float mx = wave_max(bf16_key_value(kmax));
    if (lane == 0) red_f[wv] = mx;
    __syncthreads();
    mx = red_f[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) mx = fmaxf(mx, red_f[w]);
    __syncthreads();

    // log-sum-exp in base 2
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
        __builtin_amdgcn_sched_barrier(0);
    }
    TOPK_FORGET(x);
    float sum = wave_sum(s0 + s1);
    if (lane == 0) red_f[wv] = sum;
    __syncthreads();
    sum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) sum += red_f[w];
    __syncthreads();
    const float lse = (fast_log2(sum) - c0) * CART_LN2;

    // 1. tau = K-th largest of the 1024 thread maxima (K <= 1024), bit by bit from the top, by
    // the first wavefront alone (lane l looks at maxima 16 l .. 16 l + 15): no barrier separates
    // the 16 rounds, and the other wavefronts do not spend the SIMDs' issue slots on copies of it.
    if (wv == 0) {
        uint32_t mine[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) mine[j] = reinterpret_cast<const uint32_t*>(all_kmax)[8 * lane + j];
        uint32_t t = 0;
        for (int bit = 15; bit >= 0; --bit) {
            const uint32_t cand = t | (1u << bit);
            int c = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) c += ((mine[j] & 0xffffu) >= cand) + ((mine[j] >> 16) >= cand);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, CART_WAVE);
            if (c >= K) t = cand;
        }
        if (lane == 0) tau_s = t;
    }
    __syncthreads();
    const uint32_t tau = tau_s;
    // 2. everything at or above tau goes to the list; the comparison is done on the values
    // (-0 counts as +0 there by itself), the key is formed only for what passes
    if (kmax >= tau) {
        const float tau_f = bf16_key_value(tau);
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const uint32_t w[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
            const uint32_t base = static_cast<uint32_t>(i * THREADS + tid) * 8u;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t bits = (e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16);
                if (__uint_as_float(bits) >= tau_f && base + e < static_cast<uint32_t>(V)) {
                    const int pos = atomicAdd(&list_n, 1);
                    if (pos < TOPK_CAP) { list_key[pos] = bf16_key(bits >> 16); list_idx[pos] = base + e; }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    TOPK_FORGET(x);
    __syncthreads();
    const int cnt = list_n;
    if (cnt >= K && cnt <= TOPK_CAP) {   // (cnt < K: the row has fewer than K logits above -inf)
        // 3. position of a listed logit = number of listed logits that precede it
        for (int t = tid; t < cnt; t += THREADS) {
            const uint64_t me = order_word(list_key[t], list_idx[t]);
            int rank = 0;
            for (int j = 0; j < cnt; ++j) rank += order_word(list_key[j], list_idx[j]) > me;
            if (rank < K) {
                idx_out[rank] = static_cast<int32_t>(list_idx[t]);
                logp_out[rank] = bf16_key_value(list_key[t]) - lse;
            }
        }
        return;
    }
    // the list overflowed (thousands of logits tied at the top) or came up short: K rounds over the row, re-read
    // from memory so that this rare path does not cost the common one its registers
    const bf16_t* row = logits + static_cast<size_t>(n) * V;
    select_rounds<NW>(K, red_w, [&](uint64_t prev) {
        uint64_t best = 0;
        for (int v = tid; v < V; v += THREADS) {
            const uint64_t ow = order_word(bf16_key(row[v]), static_cast<uint32_t>(v));
            if (ow < prev && ow > best) best = ow;
        }
        return best;
    }, idx_out, logp_out, lse, true);
}

// One pass over the row with 256 threads, several workgroups per CU (their memory and arithmetic
// phases overlap): log-sum-exp, and per thread its maximum and its two best logits (value and
// index).  tau = the K-th largest thread maximum as above; the list of logits >= tau is then made
// of the threads' best logits.  A thread whose second best reaches tau may hold a third: only
// such a thread reads its vectors again (about one thread per row for K = 20).  bf16 rows in
// 16-byte vectors; K <= 256.
__global__ __launch_bounds__(256) void topk_row_one_pass(const bf16_t* logits, int32_t* idx_out,
                                                         float* logp_out, int V, int K) {
    constexpr int THREADS = 256, NW = THREADS / CART_WAVE, CAP = 1024;
    __shared__ float red_max[NW], red_sum[NW];
    __shared__ uint64_t red_w[NW];
    __shared__ __align__(16) uint16_t all_kmax[THREADS];
    __shared__ uint32_t list_key[CAP];
    __shared__ uint32_t list_idx[CAP];
    __shared__ int list_n;
    __shared__ uint32_t tau_s;
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const bf16_t* row = logits + static_cast<size_t>(n) * V;
    const u32x4* src = reinterpret_cast<const u32x4*>(row);
    const int nvec = V >> 3;
    idx_out += static_cast<size_t>(n) * K;
    logp_out += static_cast<size_t>(n) * K;
    if (tid == 0) list_n = 0;

    // per thread: a running maximum (raw, as in the resident kernel), the sum of
    // 2^(x log2e - reference) against a reference that moves only in whole steps, and the two
    // best among its logits above -inf.  The two best are kept as 32-bit words, order key of the
    // value in the upper half and 0xffff - (position among the thread's own elements) in the
    // lower, so that "larger value first, then lower index" is an unsigned comparison and the
    // update is three min / max instructions per element with no branch: a vector whose maximum
    // exceeds the thread's second best is rare for a thread but not for a wavefront (some lane
    // of 64 sees one in most iterations), so the update runs almost every time and has to be cheap.
    constexpr uint32_t NONE = 0x007f0000u;           // the word of -inf at the last position: below every listed logit
    float tmax = __uint_as_float(0xff7f0000u), ref = -3.0e38f, sum = 0.f;
    uint32_t t1 = NONE, t2 = NONE;
    float t2v = __uint_as_float(0xff800000u);        // value of the second best (-inf: none)
    const float ninf = __uint_as_float(0xff800000u);
    auto take = [&](int lbase /* 0xffff - first position of the vector */, const u32x4 q) __attribute__((always_inline)) {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
        float vv = __uint_as_float(0xff800000u);     // maximum of this vector
#pragma unroll
        for (int e = 0; e < 4; ++e) vv = max3_raw(vv, w[e] & 0xffff0000u, w[e] << 16);
        if (vv > t2v) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t bits = (e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16);
                float x;     // -0 -> +0 (one value: ties go by index), NaN -> -inf (never listed)
                asm("v_add_f32 %0, 0, %1\n\tv_max_f32 %0, %0, %2" : "=&v"(x) : "v"(bits), "v"(ninf));
                const uint32_t u = __float_as_uint(x);
                const uint32_t key = u ^ (static_cast<uint32_t>(static_cast<int32_t>(u) >> 31) | 0x80000000u);
                const uint32_t wd = (key & 0xffff0000u) | static_cast<uint32_t>(lbase - e);
                const uint32_t lo = t1 < wd ? t1 : wd;
                t1 = t1 > wd ? t1 : wd;
                t2 = t2 > lo ? t2 : lo;
            }
            const uint32_t k = t2 & 0xffff0000u;
            const uint32_t m = ~static_cast<uint32_t>(static_cast<int32_t>(k) >> 31) | 0x80000000u;
            t2v = __uint_as_float((k ^ m) & 0xffff0000u);
        }
        const float vm = max3_raw(tmax, __float_as_uint(vv), __float_as_uint(vv));
        tmax = vm;
        const float need = __uint_as_float(__float_as_uint(vm) & 0xffff0000u) * CART_LOG2E;
        if (need > ref) {                      // (rare after the first few vectors)
            sum *= fast_exp2(ref - need);
            ref = need;
        }
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            s0 += fast_exp2(fmaf(__uint_as_float(w[e] << 16), CART_LOG2E, -ref));
            s1 += fast_exp2(fmaf(__uint_as_float(w[e] & 0xffff0000u), CART_LOG2E, -ref));
        }
        sum += s0 + s1;
    };
    // Four vectors per thread in flight instead of one: 3 % (1.15 -> 1.11 ms for 16384 rows of
    // 128256 logits).  At 3.8 TB/s of logits the kernel is bound by its arithmetic, one exponential
    // per logit, not by the loads.
    int v = tid, lb = 0xffff;
    for (; v + 3 * THREADS < nvec; v += 4 * THREADS, lb -= 32) {
        const u32x4 q0 = src[v], q1 = src[v + THREADS], q2 = src[v + 2 * THREADS], q3 = src[v + 3 * THREADS];
        take(lb, q0);
        take(lb - 8, q1);
        take(lb - 16, q2);
        take(lb - 24, q3);
    }
    for (; v < nvec; v += THREADS, lb -= 8) take(lb, src[v]);
    // the thread's best two as (order key, token index): position p of its own elements is
    // element p % 8 of its vector p / 8, i.e. token 8 (tid + THREADS (p / 8)) + p % 8
    const uint32_t k1 = t1 >> 16, k2 = t2 >> 16;
    const bool has1 = k1 > (NONE >> 16), has2 = k2 > (NONE >> 16);
    const uint32_t p1 = 0xffffu - (t1 & 0xffffu);
    const uint32_t idx1 = 8u * (static_cast<uint32_t>(tid) + THREADS * (p1 >> 3)) + (p1 & 7u);
    const uint32_t kmax = bf16_key(__float_as_uint(tmax) >> 16);
    all_kmax[tid] = static_cast<uint16_t>(kmax);
    const float wref = wave_max(ref);
    sum = wave_sum(sum * fast_exp2(ref - wref));
    if (lane == 0) { red_max[wv] = wref; red_sum[wv] = sum; }
    __syncthreads();
    float gref = red_max[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) gref = fmaxf(gref, red_max[w]);
    sum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) sum += red_sum[w] * fast_exp2(red_max[w] - gref);
    const float lse = (gref + fast_log2(sum)) * CART_LN2;

    // tau = K-th largest of the 256 thread maxima, by the first wavefront (4 maxima per lane)
    if (wv == 0) {
        const uint32_t m0 = reinterpret_cast<const uint32_t*>(all_kmax)[2 * lane];
        const uint32_t m1 = reinterpret_cast<const uint32_t*>(all_kmax)[2 * lane + 1];
        uint32_t t = 0;
        for (int bit = 15; bit >= 0; --bit) {
            const uint32_t cand = t | (1u << bit);
            int c = ((m0 & 0xffffu) >= cand) + ((m0 >> 16) >= cand) + ((m1 & 0xffffu) >= cand) + ((m1 >> 16) >= cand);
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, CART_WAVE);
            if (c >= K) t = cand;
        }
        if (lane == 0) tau_s = t;
    }
    __syncthreads();
    const uint32_t tau = tau_s;
    // (tau at or below -inf: fewer than K threads hold a logit above -inf; the threads' best
    // logits leave the -inf ones out, so such a row takes the selection rounds below)
    const bool listed = tau > bf16_key(0xff80u);
    if (listed) {
        if (has2 && k2 >= tau) {
            // both of the thread's best reach tau: there may be more, read its vectors again
            const float tau_f = bf16_key_value(tau);
            for (int v = tid; v < nvec; v += THREADS) {
                const u32x4 q = src[v];
                const uint32_t w[4] = {q.x, q.y, q.z, q.w};
                float vm = __uint_as_float(0xff7f0000u);
#pragma unroll
                for (int e = 0; e < 4; ++e) vm = max3_raw(vm, w[e] & 0xffff0000u, w[e] << 16);
                if (__uint_as_float(__float_as_uint(vm) & 0xffff0000u) >= tau_f) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint32_t bits = (e & 1) ? (w[e >> 1] & 0xffff0000u) : (w[e >> 1] << 16);
                        if (__uint_as_float(bits) >= tau_f) {
                            const int pos = atomicAdd(&list_n, 1);
                            if (pos < CAP) { list_key[pos] = bf16_key(bits >> 16); list_idx[pos] = 8u * v + e; }
                        }
                    }
                }
            }
        } else if (has1 && k1 >= tau) {
            const int pos = atomicAdd(&list_n, 1);
            if (pos < CAP) { list_key[pos] = k1; list_idx[pos] = idx1; }
        }
    }
    __syncthreads();
    const int cnt = list_n;
    if (listed && cnt >= K && cnt <= CAP) {
        for (int t = tid; t < cnt; t += THREADS) {
            const uint64_t me = order_word(list_key[t], list_idx[t]);
            int rank = 0;
            for (int j = 0; j < cnt; ++j) rank += order_word(list_key[j], list_idx[j]) > me;
            if (rank < K) {
                idx_out[rank] = static_cast<int32_t>(list_idx[t]);
                logp_out[rank] = bf16_key_value(list_key[t]) - lse;
            }
        }
        return;
    }
    select_rounds<NW>(K, red_w, [&](uint64_t prev) {
        uint64_t best = 0;
        for (int v = tid; v < V; v += THREADS) {
            const uint64_t ow = order_word(bf16_key(row[v]), static_cast<uint32_t>(v));
            if (ow < prev && ow > best) best = ow;
        }
        return best;
    }, idx_out, logp_out, lse, true);
}

// any vocabulary size, fp32 or bf16 logits: log-sum-exp, then K rounds straight from memory
template <typename T>
__global__ __launch_bounds__(256) void topk_row_stream(const T* logits, int32_t* idx_out, float* logp_out,
                                                       int V, int K) {
    constexpr int THREADS = 256, NW = THREADS / CART_WAVE;
    __shared__ float red_max[NW], red_sum[NW];
    __shared__ uint64_t red_w[NW];
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const T* src = logits + static_cast<size_t>(n) * V;
    idx_out += static_cast<size_t>(n) * K;
    logp_out += static_cast<size_t>(n) * K;
    float mx = -3.0e38f, sum = 0.f;
    for (int v = tid; v < V; v += THREADS) {
        const float y = elem<T>::load(src + v) * CART_LOG2E;
        const float nm = fmaxf(mx, y);
        sum = sum * fast_exp2(mx - nm) + fast_exp2(y - nm);
        mx = nm;
    }
    const float wmx = wave_max(mx);
    sum = wave_sum(sum * fast_exp2(mx - wmx));
    if (lane == 0) { red_max[wv] = wmx; red_sum[wv] = sum; }
    __syncthreads();
    float gmx = red_max[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) gmx = fmaxf(gmx, red_max[w]);
    sum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) sum += red_sum[w] * fast_exp2(red_max[w] - gmx);
    __syncthreads();
    const float lse = (gmx + fast_log2(sum)) * CART_LN2;
    select_rounds<NW>(K, red_w, [&](uint64_t prev) {
        uint64_t best = 0;
        for (int v = tid; v < V; v += THREADS) {
            const uint64_t ow = order_word(f32_key(elem<T>::load(src + v)), static_cast<uint32_t>(v));
            if (ow < prev && ow > best) best = ow;
        }
        return best;
    }, idx_out, logp_out, lse, false);
}

int launch_topk(const cart_topk_desc& d, const void* logits, int32_t* idx, float* logp, hipStream_t st) {
    trace_begin(st);   // kernel order: the row kernel
    const bool vec = d.logits_dtype == CART_BF16 && (d.V % 8) == 0;
    const bool resident = vec && d.V <= 1024 * 16 * 8 && d.K <= 1024;
#ifndef CART_TOPK_RESIDENT
#define CART_TOPK_RESIDENT 0
#endif
    if (vec && d.K <= 256 && !(CART_TOPK_RESIDENT && resident)) {
        hipLaunchKernelGGL(topk_row_one_pass, dim3(d.N), dim3(256), 0, st, static_cast<const bf16_t*>(logits), idx,
                           logp, d.V, d.K);
    } else if (resident) {
        const bf16_t* x = static_cast<const bf16_t*>(logits);
        const int nvec = d.V / 8;
        if (nvec <= 1024 * 4)
            hipLaunchKernelGGL(topk_row_resident<4>, dim3(d.N), dim3(1024), 0, st, x, idx, logp, d.V, d.K);
        else if (nvec <= 1024 * 8)
            hipLaunchKernelGGL(topk_row_resident<8>, dim3(d.N), dim3(1024), 0, st, x, idx, logp, d.V, d.K);
        else
            hipLaunchKernelGGL(topk_row_resident<16>, dim3(d.N), dim3(1024), 0, st, x, idx, logp, d.V, d.K);
    } else if (d.logits_dtype == CART_BF16) {
        hipLaunchKernelGGL(topk_row_stream<bf16_t>, dim3(d.N), dim3(256), 0, st, static_cast<const bf16_t*>(logits),
                           idx, logp, d.V, d.K);
    } else {
        hipLaunchKernelGGL(topk_row_stream<float>, dim3(d.N), dim3(256), 0, st, static_cast<const float*>(logits),
                           idx, logp, d.V, d.K);
    }
    trace_mark(st);
    return static_cast<int>(hipGetLastError());
}

}  // namespace cart
