// Two microbenchmarks that measure what this chip can actually deliver, so that the benchmark can quote roofline
// fractions against measured ceilings next to the published peaks:
//   gqla_probe_stream_read   streaming 16-byte reads of a device buffer (achievable HBM read bandwidth)
//   gqla_probe_mfma_bf16     register-resident v_mfma_f32_32x32x16_bf16 loop, one wave per SIMD on every CU, operands
//                            with random sign and mantissa bits (the matrix pipeline clocks down with toggling data,
//                            so constant operands would overstate what a real kernel can get)
// They compute nothing of the method and are only timed by the caller (events around the call).
#include "gqla_device.h"

namespace gqla {

namespace {

__global__ void __launch_bounds__(256) probe_stream_read_kernel(const u32x4* __restrict__ p, size_t n_per_block, uint32_t* sink) {
  const u32x4* q = p + (size_t)blockIdx.x * n_per_block;
  u32x4 acc = {0u, 0u, 0u, 0u};
  // four independent 16-byte loads per lane in flight; n_per_block is a multiple of 4 * 256
  for (size_t i = threadIdx.x; i < n_per_block; i += 4 * 256) {
    const u32x4 a = __builtin_nontemporal_load(q + i), b = __builtin_nontemporal_load(q + i + 256);
    const u32x4 c = __builtin_nontemporal_load(q + i + 512), d = __builtin_nontemporal_load(q + i + 768);
    acc ^= a ^ b ^ c ^ d;
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) sink[0] = acc[0];  // keeps the loads alive; practically never true
}

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7feb352dU;
  x ^= x >> 15;
  x *= 0x846ca68bU;
  x ^= x >> 16;
  return x;
}

__global__ void __launch_bounds__(256) probe_mfma_kernel(uint32_t* sink, int iters) {
  bf16x8 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    u32x4 ua, ub;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t h1 = probe_hash(threadIdx.x * 131u + blockIdx.x * 7u + j * 17u + e), h2 = probe_hash(h1 + 12345u);
      ua[e] = (h1 & 0x807f807fu) | 0x3f003f00u;  // bf16 pairs in [0.5, 1) with random sign and mantissa
      ub[e] = (h2 & 0x807f807fu) | 0x3f003f00u;
    }
    a[j] = __builtin_bit_cast(bf16x8, ua);
    b[j] = __builtin_bit_cast(bf16x8, ub);
  }
  f32x16 c0, c1, c2, c3;
#pragma unroll
  for (int i = 0; i < 16; ++i) c0[i] = c1[i] = c2[i] = c3[i] = 0.f;
  for (int i = 0; i < iters; ++i) {
    c0 = mfma32(a[0], b[0], c0);
    c1 = mfma32(a[1], b[1], c1);
    c2 = mfma32(a[2], b[2], c2);
    c3 = mfma32(a[3], b[3], c3);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == 12345.f) sink[0] = 1u;
}

}  // namespace

hipError_t launch_probe_stream_read(const void* src, size_t bytes, uint32_t* sink, int blocks, hipStream_t s) {
  const size_t n_per_block = bytes / 16 / blocks;
  probe_stream_read_kernel<<<blocks, 256, 0, s>>>((const u32x4*)src, n_per_block, sink);
  return hipGetLastError();
}

hipError_t launch_probe_mfma(uint32_t* sink, int iters, int blocks, hipStream_t s) {
  probe_mfma_kernel<<<blocks, 256, 0, s>>>(sink, iters);
  return hipGetLastError();
}

}  // namespace gqla
