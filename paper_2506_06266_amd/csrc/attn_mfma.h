// Building blocks of the bf16 MFMA attention kernels (gfx950, head_dim 128).
//
// Matrix-core instruction used throughout: v_mfma_f32_32x32x16_bf16, D(32x32) += A(32x16) B(16x32).
//   A: lane l holds row l%32,    k = 8*(l/32) + [0,8)      (8 bf16, 4 VGPRs)
//   B: lane l holds column l%32, k = 8*(l/32) + [0,8)
//   D: lane l holds column l%32, rows 8*(r/4) + 4*(l/32) + r%4 for r in [0,16)
// Every product here is arranged so that the index kept per lane (a query, or a key) is the D
// column and the contracted index of the NEXT product is the D row; the fp32 tile then turns
// into the next product's 16-bit operand inside the lane, with no LDS round trip.  The D-row
// order is a permutation of the contracted index; the other operand is fetched from LDS in the
// same permuted order (see k_slot_row below), which a sum does not mind.
#pragma once

#include <type_traits>
#include <utility>

#include "cart_common.h"

namespace cart {
namespace mfma {

// compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{})
template <typename F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

// Masking without compares: entry r of a score block (D row 8 (r/4) + r%4 + 4 g, g folded into
// thr by the caller) is hidden when its row exceeds thr (mask_above) or lies below it
// (mask_below).  bound_r = (thr - row + 1/2) * 1e30 is far above every score where the entry is
// visible and far below where it is hidden, so x = min(x, bound_r) does the job in two plain
// vector instructions per entry, with no condition registers between them (the compare / select
// form goes through scalar registers and costs several times more).  A hidden entry ends up at
// -5e29 or below: its exponential is an exact 0.
__device__ __forceinline__ float vmin_raw(float a, float b) {
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
template <typename V16>
__device__ __forceinline__ void mask_above(V16& x, int thr) {
    const int t = min(max(thr, -64), 64);
    const float tf = fmaf(static_cast<float>(t), 1.0e30f, 0.5e30f);
#pragma unroll
    for (int r = 0; r < 16; ++r) x[r] = vmin_raw(x[r], tf - static_cast<float>(8 * (r >> 2) + (r & 3)) * 1.0e30f);
}
template <typename V16>
__device__ __forceinline__ void mask_below(V16& x, int thr) {
    const int t = min(max(thr, -64), 64);
    const float tf = fmaf(static_cast<float>(-t), 1.0e30f, 0.5e30f);
#pragma unroll
    for (int r = 0; r < 16; ++r) x[r] = vmin_raw(x[r], tf + static_cast<float>(8 * (r >> 2) + (r & 3)) * 1.0e30f);
}

// Rows of sequence b, and where the per-row statistics (lse, delta) of its heads live: the value
// of token i of head h is at stat_b + h * stat_h + i.
//   batched layout (cu == nullptr): rows b*S .. b*S+S-1 of [B,S,...]; statistics [B,Hq,S]
//   packed layout: rows cu[b] .. cu[b+1]-1 of [T,...];                statistics [Hq,T]
struct SeqSpan { size_t t0; size_t stat_b; size_t stat_h; int len; };
__device__ __forceinline__ SeqSpan seq_span(const int32_t* cu, int b, int T, int S, int Hq) {
    SeqSpan sp;
    if (cu) {
        const int c0 = cu[b];
        sp.t0 = static_cast<size_t>(c0);
        sp.len = cu[b + 1] - c0;
        sp.stat_b = sp.t0;
        sp.stat_h = static_cast<size_t>(T);
    } else {
        sp.t0 = static_cast<size_t>(b) * S;
        sp.len = S;
        sp.stat_b = static_cast<size_t>(b) * Hq * S;
        sp.stat_h = static_cast<size_t>(S);
    }
    return sp;
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int HD = 128;           // head_dim
constexpr int ROW_B = HD * 2;     // bytes per key/value/query row, in global memory and in LDS
constexpr float NEG_BIG = -1.0e30f;
constexpr float RESCALE_GAP = 8.0f;   // running max is moved only when exceeded by 2^8

__device__ __forceinline__ f32x16 mma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// The same product with the result in ordinary vector registers (the compiler's own choice for
// the builtin is an accumulation register whenever a kernel uses those at all) and the B operand
// read from an accumulation register.  The compiler does not know these are matrix-core
// instructions: a consumer on the vector ALU must be at least 20 wait states away.
// Where that distance comes from, kernel by kernel (a product occupies the matrix cores for 32
// cycles, so one product issued in between already covers it; every place states its own margin):
//   forward        S(u+1) written in groups 0-15 of an iteration, first read by the vector ALU
//                  in group 0 of the next one: the 16 O products of groups 16-31 lie between.
//   dQ             block 1's S / dP written up to groups 44 / 45, first read in group 0 of the
//                  next iteration: 3 products between (groups 46, 47, 0); block 0's written up to
//                  groups 46 / 47, first read in group 16: 17 products between.  The masked path
//                  reads them at the top of the iteration and waits 24 states first.
//   dK + dV, A     S(u+1) written in groups 0-15, first read in group 0 of the next iteration:
//                  the 16 dV products between.
//   dK + dV, B     dP(u) written in groups 0-15, first read in group 4 of the next iteration: the
//                  16 dK products and 4 more between.
//   prologues      every first score product is followed by s_nop 15; s_nop 7 (24 states).
// The GPU tests hold the tripwires: the forward and the backward run twice bit-equal, and the
// matrix-core kernels against the vector kernels and the oracle over a sweep of random shapes.
__device__ __forceinline__ void mma_vd_zero(f32x16& d, bf16x8 a, const u32x4& b) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
}
// d = a b + init (init in its own registers, left unchanged)
__device__ __forceinline__ void mma_vd_first(f32x16& d, bf16x8 a, const u32x4& b, const f32x16& init) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(d) : "v"(a), "a"(b), "v"(init));
}
__device__ __forceinline__ void mma_vd(f32x16& d, bf16x8 a, const u32x4& b) {
    asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
}

// LDS tiles are [rows][128] bf16, 256 bytes per row, unpadded; the 16-byte chunk c of row r is
// stored at chunk position c ^ swz(r).  swz is a bijection of r % 16 (16 consecutive rows read
// at one logical chunk hit 16 distinct positions: row-wise ds_read_b128 is conflict-free) whose
// bits 2..3 are r % 4 (4 consecutive rows x 4 consecutive chunks cover all 16 positions: the
// transposing read is conflict-free too).
__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// row-wise operand fragment: the 8 bf16 at columns [col, col+8) of one row (col % 8 == 0)
__device__ __forceinline__ bf16x8 lds_frag_n(const char* tile, int row, int col) {
    return *reinterpret_cast<const bf16x8*>(tile + row * ROW_B + (((col >> 3) ^ swz(row)) << 4));
}

// Transposed operand fragment for one 16-deep k-step of a [k][n] row-major tile: the lane that
// owns operand row/column n gets the 8 k-values whose k-slots match the D-row order above:
// slots e = 0..3 -> k = k0 + 4g + e, slots 4..7 -> k = k0 + 8 + 4g + (e-4), g = lane/32.
// ds_read_b64_tr_b16: within each block of 16 lanes, lane i receives, for e = 0..3, element i%4 of
// the 8 bytes addressed by lane 4e + i/4; so lane s of a block addresses row k + s/4, columns
// n0 + 4*(s%4) .. +3, and lane i ends up with column n0 + i of rows k .. k+3.
__device__ __forceinline__ bf16x8 lds_frag_t(const char* tile, int k0, int n0, int lane) {
    const int blk = lane >> 4, s = lane & 15, g = lane >> 5;
    const int row = k0 + 4 * g + (s >> 2);
    const int col = n0 + 16 * (blk & 1) + 4 * (s & 3);
    const int half = ((col >> 2) & 1) * 8;
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_ptr)(tile + row * ROW_B + (((col >> 3) ^ swz(row)) << 4) + half));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_ptr)(tile + (row + 8) * ROW_B + (((col >> 3) ^ swz(row + 8)) << 4) + half));
    s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

// The same two fragment kinds from precomputed 32-bit LDS byte addresses (per-lane part computed
// once, compile-time offsets added at the use): frag_n_ofs / frag_t_ofs give the per-lane offset
// of a fragment inside a tile whose first row is a multiple of 16.
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint32_t frag_n_ofs(int lane, int t8) {
    const int lc = lane & 31, lg = lane >> 5;
    return lc * ROW_B + (((2 * t8 + lg) ^ swz(lc)) << 4);
}
__device__ __forceinline__ void frag_t_ofs(int lane, int db, uint32_t& lo, uint32_t& hi) {
    const int s = lane & 15, g = lane >> 5;
    const int row = 4 * g + (s >> 2);
    const int col = 32 * db + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    const int half = ((col >> 2) & 1) * 8;
    lo = row * ROW_B + (((col >> 3) ^ swz(row)) << 4) + half;
    hi = (row + 8) * ROW_B + (((col >> 3) ^ swz(row + 8)) << 4) + half;
}
__device__ __forceinline__ bf16x8 lds_ld_frag(uint32_t addr) {
    return *(const bf16x8 __attribute__((address_space(3)))*)addr;
}
__device__ __forceinline__ f32x4 lds_ld_f32x4(uint32_t addr) {
    return *(const f32x4 __attribute__((address_space(3)))*)addr;
}
__device__ __forceinline__ bf16x8 lds_ld_frag_t(uint32_t lo, uint32_t hi) {
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)lo);
    const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)hi);
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7));
}

// D row held in register r of lane-group g (the k index the next product contracts over)
__device__ __forceinline__ int d_row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

// value held by the lane 32 away
__device__ __forceinline__ float partner(float x) {
    uint32_t u = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}
__device__ __forceinline__ float partner_max(float x) {
    uint32_t u = __float_as_uint(x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// 8 fp32 D registers [r0, r0+8) -> one 16-bit operand fragment (same lane, same column)
__device__ __forceinline__ bf16x8 pack_frag(const f32x16& s, int r0) {
    u32x4 w = {pack_bf16x2(s[r0 + 0], s[r0 + 1]), pack_bf16x2(s[r0 + 2], s[r0 + 3]),
               pack_bf16x2(s[r0 + 4], s[r0 + 5]), pack_bf16x2(s[r0 + 6], s[r0 + 7])};
    return __builtin_bit_cast(bf16x8, w);
}

// ---- direct-to-LDS loads --------------------------------------------------------------------
// The loads are written as inline assembly so that the wait for them sits where the pipeline
// wants it (one s_waitcnt vmcnt(0) in front of the barrier that publishes the tile, a whole
// iteration after the loads went out) and not in front of the next LDS read of any address.
// M0 carries the wave-uniform LDS byte address; lane i's 16 (4) bytes land at M0 + 16 i (4 i).
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((const __attribute__((address_space(3))) void*)p));
}
// base: wave-uniform global address; voff: per-lane unsigned byte offset from it
__device__ __forceinline__ void dma16(const char* base, uint32_t voff, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(base), "s"(lds) : "memory", "m0");
}
__device__ __forceinline__ void dma4(const char* base, uint32_t voff, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :: "v"(voff), "s"(base), "s"(lds) : "memory", "m0");
}
// every direct-to-LDS load of this wavefront has landed
__device__ __forceinline__ void dma_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// all but the wavefront's N most recent direct-to-LDS loads have landed
template <int N>
__device__ __forceinline__ void dma_wait_but() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

// Tile of ROWS rows x 256 bytes -> LDS (row r at 256 r, 16-byte chunks swizzled), cooperatively
// by the 4 wavefronts of a 256-thread workgroup.  One load instruction moves 64 chunks = 4 tile
// rows; lane i's chunk lands at (wave-uniform base) + 16 i, so the lane fetches the logical
// chunk that belongs at that position under the swizzle.  Tile row r comes from tensor row
// min(j0 + r, last) of a slice that starts at `base` with `pitch` bytes between rows (base, j0,
// last, pitch wave-uniform; j0 <= last; rows past `last` repeat it and are masked by the
// caller, so their contents never reach a result; 64 * pitch < 2^32).
template <int ROWS>
__device__ __forceinline__ void tile_load_async(char* tile, const char* base, int j0, int last, uint32_t pitch) {
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int PER_WAVE = ROWS / 16;      // instructions per wavefront
    const char* tb = base + static_cast<size_t>(j0) * pitch;
    const int lim = last - j0;
    const uint32_t lds0 = lds_addr(tile);
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
        const int r0 = (PER_WAVE * wv + i) * 4;
        const int r = r0 + (lane >> 4);
        const uint32_t voff = static_cast<uint32_t>(min(r, lim)) * pitch + (((lane & 15) ^ swz(r)) << 4);
        dma16(tb, voff, lds0 + r0 * ROW_B);
    }
}

}  // namespace mfma
}  // namespace cart
