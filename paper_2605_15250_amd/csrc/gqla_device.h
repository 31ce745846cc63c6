// Device-side helpers shared by the gfx950 kernels: MFMA fragment types, wave64 half swaps,
// cache address arithmetic.  Lane layouts used throughout (wave64, v_mfma_f32_32x32x16_bf16):
//   A fragment  lane l holds A[m = l % 32][k = 8*(l / 32) + 0..7]
//   B fragment  lane l holds B[k = 8*(l / 32) + 0..7][n = l % 32]
//   C fragment  lane l, register i holds C[m = 8*(i / 4) + 4*(l / 32) + i % 4][n = l % 32]
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "gqla_internal.h"

// Names of all 256 accumulation registers, for the clobber list of kernels that address them by name in inline
// assembly (the compiler then counts them as used and keeps its own values out of them).
#define GQLA_A10(p) "a" #p "0", "a" #p "1", "a" #p "2", "a" #p "3", "a" #p "4", "a" #p "5", "a" #p "6", "a" #p "7", "a" #p "8", "a" #p "9"
#define GQLA_ALL_AGPRS                                                                                                   \
  "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", GQLA_A10(1), GQLA_A10(2), GQLA_A10(3), GQLA_A10(4),       \
      GQLA_A10(5), GQLA_A10(6), GQLA_A10(7), GQLA_A10(8), GQLA_A10(9), GQLA_A10(10), GQLA_A10(11), GQLA_A10(12),        \
      GQLA_A10(13), GQLA_A10(14), GQLA_A10(15), GQLA_A10(16), GQLA_A10(17), GQLA_A10(18), GQLA_A10(19), GQLA_A10(20),  \
      GQLA_A10(21), GQLA_A10(22), GQLA_A10(23), GQLA_A10(24), "a250", "a251", "a252", "a253", "a254", "a255"

namespace gqla {

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), straight-line code from the start
// (register arrays indexed by the counter are then promoted to registers even when the body is large)
template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

// Chunk partials of the 16-bit MQA-absorb decode: 8-dim vectors (16 bytes) ordered [chunk][block of 32 rows][r_kv / 8][row
// in the block].  The decode kernels' lanes (row n, four of a vector's dims per half-wave) and the combine kernel's lanes
// (row n, vector h of a k-step) then both touch contiguous memory with consecutive n.  Index of vector `vec` of row `rho`.
__device__ __forceinline__ int64_t part_vec_index(int64_t chunk, int rho, int M, int vecs_per_row, int vec) {
  const int row_blocks = (M + 31) >> 5;
  return (((chunk * row_blocks + (rho >> 5)) * vecs_per_row + vec) << 5) + (rho & 31);
}

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short i16x4;

#define GQLA_NEG_INF (-__builtin_inff())
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Two floats -> packed bf16 pair (round to nearest even), low half = a.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
  return __builtin_bit_cast(float, bits16 << 16);
}

// Exchange between the two 32-lane halves: returns {lower-half view, upper-half view}:
//   r[0] = lanes 0..31 keep x, lanes 32..63 receive y of lane-32;   r[1] = lanes 0..31 receive x of lane+32, lanes 32..63 keep y.
__device__ __forceinline__ void half_swap(uint32_t x, uint32_t y, uint32_t& r0, uint32_t& r1) {
  auto r = __builtin_amdgcn_permlane32_swap(x, y, false, false);
  r0 = r[0];
  r1 = r[1];
}

// max / sum of a value over the two lanes (l, l ^ 32).
__device__ __forceinline__ float pair_max(float v) {
  uint32_t a, b;
  uint32_t u = __builtin_bit_cast(uint32_t, v);
  half_swap(u, u, a, b);
  return fmaxf(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b));
}
__device__ __forceinline__ float pair_sum(float v) {
  uint32_t a, b;
  uint32_t u = __builtin_bit_cast(uint32_t, v);
  half_swap(u, u, a, b);
  return __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Four fp32 values -> four E4M3 codes of x * inv_scale (OCP 8-bit float, "FN" variant), round to nearest even; magnitudes
// above 448 saturate (the conversion instruction alone would turn them into NaN).  Byte k of the result is value k.
__device__ __forceinline__ uint32_t quantize_e4m3x4(float a, float b, float c, float d, float inv_scale) {
  auto q = [&](float x) { return __builtin_amdgcn_fmed3f(x * inv_scale, -448.f, 448.f); };  // clamp in one instruction
  int w = __builtin_amdgcn_cvt_pk_fp8_f32(q(a), q(b), 0, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(q(c), q(d), w, true);
  return (uint32_t)w;
}
// the value a float has after one rounding to bf16 (what a 16-bit cache would hold)
__device__ __forceinline__ float round_to_bf16(float x) { return bf16_bits_to_float(pack_bf16(x, 0.f) & 0xffffu); }
// the same for two values with one conversion instruction
__device__ __forceinline__ void round_to_bf16x2(float& x, float& y) {
  const uint32_t w = pack_bf16(x, y);
  x = __builtin_bit_cast(float, w << 16);
  y = __builtin_bit_cast(float, w & 0xffff0000u);
}

// Page id of logical page p of sequence b, or -1 when the table entry is outside the pool.
// A logical page outside the sequence's table row (a device-side length beyond max_pages * page_size) is -1 as well:
// the row of the table is never read past its end, and without a table no page of the next sequence is formed.
__device__ __forceinline__ int32_t page_of(const CacheView& c, int32_t b, int32_t p) {
  if ((uint32_t)p >= (uint32_t)c.max_pages) return -1;
  int32_t pg = c.page_table ? c.page_table[(int64_t)b * c.max_pages + p] : b * c.max_pages + p;
  return ((uint32_t)pg < (uint32_t)c.num_pages) ? pg : -1;
}

}  // namespace gqla
