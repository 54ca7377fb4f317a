// Device-side helpers shared by the gfx950 kernels of libcartridge: bf16 <-> fp32 conversion,
// wavefront (64-lane) reductions, and the internal launch prototypes the C-ABI layer calls.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/cartridge.h"

#define CART_WAVE 64
#define CART_LOG2E 1.4426950408889634f
#define CART_LN2 0.6931471805599453f

namespace cart {

typedef uint16_t bf16_t;   // raw bfloat16 bits
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_to_f32(bf16_t x) {
    return __uint_as_float(static_cast<uint32_t>(x) << 16);
}

// round-to-nearest-even; NaN stays NaN (quiet)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<bf16_t>(u >> 16);
}

// two fp32 -> packed bf16x2 (lo in bits 0..15), nearest-even, through the hardware converter
typedef __bf16 bf16x2_v __attribute__((ext_vector_type(2)));
typedef float float2_v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    float2_v f = {lo, hi};
    bf16x2_v b = __builtin_convertvector(f, bf16x2_v);
    return __builtin_bit_cast(uint32_t, b);
}

template <typename T> struct elem;
template <> struct elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, CART_WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, CART_WAVE));
    return v;
}

// Benchmark hook (cart_trace_events): records the next event of the caller's array on `st`.
struct Trace {
    void* const* events = nullptr;
    int count = 0;
    int next = 0;
};
Trace& trace();
inline void trace_begin(hipStream_t st) {
    Trace& t = trace();
    t.next = 0;
    if (t.events && t.count > 0) { hipEventRecord(static_cast<hipEvent_t>(t.events[0]), st); t.next = 1; }
}
inline void trace_mark(hipStream_t st) {
    Trace& t = trace();
    if (t.events && t.next < t.count) hipEventRecord(static_cast<hipEvent_t>(t.events[t.next++]), st);
}

// ---- internal launchers (host side), one per kernel family; all return hipError_t as int ----
int launch_kl(const cart_kl_desc& d, const void* logits, const int32_t* idx, const float* logp,
              float* loss, void* d_logits, float* row_kl, void* ws, hipStream_t st);

int launch_attn_fwd_vector(const cart_attn_desc& d, float scale, const void* q, const void* k,
                           const void* v, const void* zk, const void* zv, void* o, float* lse,
                           hipStream_t st);
int launch_attn_bwd_vector(const cart_attn_desc& d, float scale, const void* q, const void* k,
                           const void* v, const void* zk, const void* zv, const void* o,
                           const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                           float* dzk, float* dzv, void* ws, hipStream_t st);
int launch_decode_vector(const cart_decode_desc& d, float scale, const void* q, const void* zk,
                         const void* zv, const void* k, const void* v, const int32_t* cu,
                         void* o, float* lse, hipStream_t st);

// MFMA (bf16, head_dim 128) kernels
bool attn_mfma_supported(const cart_attn_desc& d);       // forward
bool attn_mfma_bwd_supported(const cart_attn_desc& d);
size_t attn_mfma_fwd_workspace(const cart_attn_desc& d, int T = 0);        // T > 0: packed rows
int launch_row_lo(const int32_t* cu, int B, int T, int32_t* row_lo, hipStream_t st);
size_t attn_mfma_bwd_workspace(const cart_attn_desc& d, long tokens = -1);   // beyond the delta array
int launch_attn_fwd_mfma(const cart_attn_desc& d, float scale, const void* q, const void* k,
                         const void* v, const void* zk, const void* zv, void* o, float* lse,
                         void* ws, hipStream_t st, const int32_t* cu = nullptr, int T = 0);
int launch_attn_bwd_mfma(const cart_attn_desc& d, float scale, const void* q, const void* k,
                         const void* v, const void* zk, const void* zv, const void* o,
                         const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                         float* dzk, float* dzv, void* ws, hipStream_t st, const int32_t* cu = nullptr,
                         int T = 0);
int launch_topk(const cart_topk_desc& d, const void* logits, int32_t* idx, float* logp, hipStream_t st);
bool decode_composed_supported(const cart_decode_composed_desc& d);
size_t decode_composed_workspace(const cart_decode_composed_desc& d, const cart_segment* shared);
int launch_decode_composed(const cart_decode_composed_desc& d, float scale, const void* q,
                           const cart_segment* shared, const void* pool_k, const void* pool_v,
                           const int32_t* cart_id, const void* k, const void* v, const int32_t* cu, void* o,
                           float* lse, void* ws, hipStream_t st);
bool decode_mfma_supported(const cart_decode_desc& d);
size_t decode_mfma_workspace(const cart_decode_desc& d);
size_t decode_static_capacity();      // bytes of the library's own per-GPU decode scratch array
void* decode_static_scratch();        // its address on the current device (nullptr on failure)
int launch_decode_mfma(const cart_decode_desc& d, float scale, const void* q, const void* zk,
                       const void* zv, const void* k, const void* v, const int32_t* cu, void* o,
                       float* lse, void* ws, hipStream_t st);

}  // namespace cart
