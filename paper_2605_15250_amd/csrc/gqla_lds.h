// LDS staging of row-major bf16 matrices for MFMA operands on gfx950.
//
// A staged matrix is a linear array of rows of ROW_CHUNKS 16-byte chunks; chunk c of row r is stored at chunk
// position c ^ (r & 7) of that row, which spreads both access patterns below over the LDS banks:
//   row_frag  lane (m = l % 32, h = l / 32) reads 8 consecutive elements of row m (an A or B fragment whose
//             contraction index runs along the row)                                   -> ds_read_b128
//   tr_frag   the contraction index runs DOWN the rows: each lane needs 2 x 4 consecutive rows of one column;
//             ds_read_b64_tr_b16 transposes 4x4 blocks among 16 lanes: lane 4q+r' of a 16-lane group receives
//             element r' of the 8-byte vectors addressed by lanes q, 4+q, 8+q, 12+q of the group.
// Rows are filled with global_load_lds_dwordx4 (HBM/L2 -> LDS without passing through VGPRs).
#pragma once

#include "gqla_device.h"

namespace gqla {

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(1))) const void* gbl_ptr_t;

// Asynchronously stage rows [0, rows_valid) of a row-major global matrix (row stride gstride bytes) and zero
// rows [rows_valid, rows_total).  Work is spread over n_waves waves; every wave of the workgroup must call it.
// Completion: s_waitcnt vmcnt(0) lgkmcnt(0) by each wave, then a workgroup barrier.
template <int ROW_CHUNKS>
__device__ __forceinline__ void stage_rows(char* lds, const char* g, int64_t gstride, int rows_total, int rows_valid,
                                           int wave, int n_waves, int lane) {
  const int n_inst = rows_total * ROW_CHUNKS / 64;
  for (int it = wave; it < n_inst; it += n_waves) {
    const int q = it * 64 + lane;
    const int row = q / ROW_CHUNKS;
    const int pos = q - row * ROW_CHUNKS;
    const int c = pos ^ (row & 7);
    if (row < rows_valid) {
      __builtin_amdgcn_global_load_lds((gbl_ptr_t)(g + (int64_t)row * gstride + c * 16), (lds_ptr_t)(lds + it * 1024),
                                       16, 0, 0);
    } else {
      *(u32x4*)(lds + q * 16) = u32x4{0u, 0u, 0u, 0u};
    }
  }
}

__device__ __forceinline__ void wait_all_memory() { __builtin_amdgcn_s_waitcnt(0); }

// 8 consecutive elements (chunk `chunk`) of row `row`.
template <int ROW_CHUNKS>
__device__ __forceinline__ bf16x8 row_frag(const char* lds, int row, int chunk) {
  return *(const bf16x8*)(lds + row * (ROW_CHUNKS * 16) + ((chunk ^ (row & 7)) << 4));
}

// Transposed fragment: lane l of the wave receives column (col0 + l % 32) of rows row_a + 0..3 (elements 0..3)
// and row_b + 0..3 (elements 4..7), where row_a / row_b are per-lane-half bases supplied by the caller
// (typically base + 8 * (l / 32) and that + 4, or any other pairing that matches the other MFMA operand).
// col0 must be a multiple of 32; row_a, row_b multiples of 4.
template <int ROW_CHUNKS>
__device__ __forceinline__ bf16x8 tr_frag(const char* lds, int row_a, int row_b, int col0, int lane) {
  const int i16 = lane & 15;
  const int e = i16 >> 2, q = i16 & 3;            // this lane ADDRESSES row (+e), columns 4q..4q+3 of its 16-col block
  const int col = col0 + ((lane >> 4) & 1) * 16 + 4 * q;
  const int chunk = col >> 3, sub = (col & 7) * 2;
  const int ra = row_a + e, rb = row_b + e;
  const char* pa = lds + ra * (ROW_CHUNKS * 16) + ((chunk ^ (ra & 7)) << 4) + sub;
  const char* pb = lds + rb * (ROW_CHUNKS * 16) + ((chunk ^ (rb & 7)) << 4) + sub;
  i16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)pa);
  i16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)pb);
  typedef __attribute__((ext_vector_type(8))) short i16x8;
  i16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

}  // namespace gqla
