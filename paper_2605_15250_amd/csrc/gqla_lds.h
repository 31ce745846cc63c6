// LDS staging of row-major bf16 matrices for MFMA operands on gfx950.
//
// Panel layout.  A staged matrix of R rows and 8*NP 16-byte chunks per row is kept as NP panels of [R][128 bytes]:
// chunk c of row r lives in panel c / 8 at byte  r*128 + (((c & 7) ^ swz(r)) << 4),  swz(r) = (r >> 1) & 7.
// The XOR spreads both access patterns below over the LDS banks:
//   row fragment         lane (m = l % 32, h = l / 32) reads 8 consecutive elements of row m (an MFMA operand whose
//                        contraction index runs along the row)                                  -> ds_read_b128
//   transposed fragment  the contraction index runs DOWN the rows: each lane needs 2 x 4 consecutive rows of one
//                        column.  ds_read_b64_tr_b16 transposes 4x4 blocks among 16 lanes: lane 4q+r' of a 16-lane
//                        group receives element r' of the 8-byte vectors addressed by lanes q, 4+q, 8+q, 12+q.
// Panels are filled with global_load_lds_dwordx4 (HBM/L2 -> LDS without passing through VGPRs): one wave
// instruction moves 8 rows x 128 bytes, i.e. 1 KB that is contiguous in the panel.
#pragma once

#include "gqla_device.h"

namespace gqla {

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(1))) const void* gbl_ptr_t;
typedef __attribute__((ext_vector_type(8))) short i16x8;

__device__ __forceinline__ int lds_swz(int row) { return (row >> 1) & 7; }

// Staging of a whole matrix with ROWS rows of NP*128 bytes (row stride GSTRIDE bytes) by the NWAVES waves of a
// workgroup (NWAVES even and dividing ROWS/8).  Completion: s_waitcnt vmcnt(..) by each wave, then a workgroup barrier.
template <int ROWS, int NP, int NWAVES, int GSTRIDE>
__device__ __forceinline__ uint32_t stage_lane_offset(int wave, int lane) {
  const int row0 = 8 * wave + (lane >> 3);
  const int c = (lane & 7) ^ ((4 * wave + (lane >> 4)) & 7);
  return row0 * GSTRIDE + c * 16;
}
// g and wave must be wave-uniform; lane_off = stage_lane_offset(wave, lane) is the only per-lane part of the address.
// The instruction is written as inline assembly on purpose: the compiler then does not know that LDS is being written
// behind its back, and does not put a "wait for every outstanding load" in front of the next LDS read (it cannot see
// that the reads go to another buffer).  The caller orders things itself: s_waitcnt vmcnt(0) and a workgroup barrier
// before the staged tile is read.
// STREAM: the source is read once (a cache tile): the request carries the non-temporal hint, which on this chip
// raises the rate at which LDS-DMA streams from HBM from 6.0 to 6.8 TB/s (own probe: 256 workgroups of 4 waves, ring
// of four 36 KB buffers; the number of tiles in flight made no difference).
template <int ROWS, int NP, int NWAVES, int GSTRIDE, bool STREAM = false>
__device__ __forceinline__ void stage_panels_step(char* lds, const char* g, int wave, uint32_t lane_off, int u) {
  static_assert(NWAVES % 2 == 0 && (ROWS / 8) % NWAVES == 0, "wave count must be even and divide ROWS/8");
  constexpr int K = ROWS / 8 / NWAVES;
  const int a = u / K, v = u % K;
  const char* base = g + (8 * NWAVES * v * GSTRIDE + a * 128);
  const uint32_t dst = (uint32_t)(uintptr_t)(lds_ptr_t)(lds + a * (ROWS * 128) + (wave + NWAVES * v) * 1024);
  if constexpr (STREAM)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" : : "s"(dst), "v"(lane_off), "s"(base) : "memory");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(dst), "v"(lane_off), "s"(base)
               : "memory");  // M0 is written here.  It cannot be named as a clobber (the compiler treats it as reserved and
                             // warns that such a clobber is not honoured); the kernels that use these blocks contain
                             // nothing for which the compiler itself needs M0 (no LDS-DMA builtin, no indirect register
                             // indexing, no messages), and every block sets M0 before it uses it.
}

// Whole matrix (all ROWS rows present), this wave's share in one burst of asm steps.
template <int ROWS, int NP, int NWAVES, int GSTRIDE, bool STREAM = false>
__device__ __forceinline__ void stage_panels_full(char* lds, const char* g, int wave, int lane) {
  const uint32_t lane_off = stage_lane_offset<ROWS, NP, NWAVES, GSTRIDE>(wave, lane);
#pragma unroll
  for (int u = 0; u < NP * (ROWS / 8 / NWAVES); ++u) stage_panels_step<ROWS, NP, NWAVES, GSTRIDE, STREAM>(lds, g, wave, lane_off, u);
}

__device__ __forceinline__ void wait_all_memory() { __builtin_amdgcn_s_waitcnt(0); }

// 8 consecutive elements (chunk `chunk`) of row `row` of a staged matrix with ROWS rows.
template <int ROWS>
__device__ __forceinline__ bf16x8 row_frag(const char* lds, int row, int chunk) {
  return *(const bf16x8*)(lds + (chunk >> 3) * (ROWS * 128) + row * 128 + (((chunk & 7) ^ lds_swz(row)) << 4));
}

// Transposed fragment: lane l receives column (col0 + l % 32) of rows row_a + 0..3 (elements 0..3) and row_b + 0..3
// (elements 4..7); row_a, row_b are per-lane-half values supplied by the caller (multiples of 4), col0 a multiple of 32.
template <int ROWS>
__device__ __forceinline__ bf16x8 tr_frag(const char* lds, int row_a, int row_b, int col0, int lane) {
  const int i16 = lane & 15;
  const int e = i16 >> 2, q = i16 & 3;  // this lane ADDRESSES row (+e), columns 4q..4q+3 of its 16-column block
  const int col = col0 + ((lane >> 4) & 1) * 16 + 4 * q;
  const int chunk = col >> 3, sub = (col & 7) * 2;
  const int ra = row_a + e, rb = row_b + e;
  const char* panel = lds + (chunk >> 3) * (ROWS * 128) + sub;
  const char* pa = panel + ra * 128 + (((chunk & 7) ^ lds_swz(ra)) << 4);
  const char* pb = panel + rb * 128 + (((chunk & 7) ^ lds_swz(rb)) << 4);
  const i16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)pa);
  const i16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)pb);
  const i16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// Transposed fragments in natural contraction order out of a staged [ROWS][NP*64] matrix: fragment (ks, mt) holds,
// for column 32*mt + l % 32, rows 16*ks + 8*(l / 32) + 0..7.  The per-lane part of the two read addresses depends only
// on the parity of mt (the swizzle flips the 64-byte half with the lane half), so four lane offsets cover the
// whole matrix and everything else is a compile-time offset:  base[read][mt & 1] + (mt >> 1)*ROWS*128 + ks*2048.
struct TrNatural {
  uint32_t base[2][2];
};

__device__ __forceinline__ TrNatural make_tr_natural(int lane) {
  const int h = lane >> 5, i16 = lane & 15, e = i16 >> 2, q = i16 & 3, g1 = (lane >> 4) & 1;
  const int cl = 2 * g1 + (q >> 1), sub = (q & 1) * 8;
  TrNatural t;
#pragma unroll
  for (int rd = 0; rd < 2; ++rd) {
    const int x = 2 * rd + (e >> 1);  // low swizzle bits of row 16*ks + 8*h + e + 4*rd; bit 2 of the swizzle is h
#pragma unroll
    for (int par = 0; par < 2; ++par)
      t.base[rd][par] = (8 * h + e + 4 * rd) * 128 + ((4 * (par ^ h) + (cl ^ x)) << 4) + sub;
  }
  return t;
}

template <int ROWS>
__device__ __forceinline__ bf16x8 tr_natural_frag(const char* lds, const TrNatural& t, int ks, int mt) {
  const int off = (mt >> 1) * (ROWS * 128) + ks * 2048;
  const i16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(lds + t.base[0][mt & 1] + off));
  const i16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(lds + t.base[1][mt & 1] + off));
  const i16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

}  // namespace gqla
