// Cache switch 16-bit expanded cache -> 8-bit expanded cache (K_C and V as E4M3 codes, k_R copied).
// The paper lists quantised KV caches as complementary to the method and leaves them out of its model (Sec. 2;
// Sec. 5.1, item (i)); the format is this library's (see gqla.h): every 16-byte vector of the two planes holds what
// one lane of a 32x32x16 MFMA consumes in two consecutive k-steps, so the decode needs half the load instructions.
//   code = E4M3(fp32(x) * inv_scale), round to nearest even, magnitudes above 448 saturate (the conversion
//   instruction alone would turn them into NaN).
#include "gqla_device.h"

namespace gqla {

namespace {

// 8 bf16 (one 16-byte vector) -> 8 codes (two words)
__device__ __forceinline__ u32x2 e4m3x8(u32x4 v, float inv_scale) {
  uint32_t lo, hi;
  lo = quantize_e4m3x4(bf16_bits_to_float(v[0] & 0xffffu), bf16_bits_to_float(v[0] >> 16), bf16_bits_to_float(v[1] & 0xffffu),
              bf16_bits_to_float(v[1] >> 16), inv_scale);
  hi = quantize_e4m3x4(bf16_bits_to_float(v[2] & 0xffffu), bf16_bits_to_float(v[2] >> 16), bf16_bits_to_float(v[3] & 0xffffu),
              bf16_bits_to_float(v[3] >> 16), inv_scale);
  return u32x2{lo, hi};
}

// One workgroup per (logical page, sequence).  Only bytes that belong to tokens t < L_b are written.
template <int DH, int DR>
__global__ void __launch_bounds__(256) quantize_expanded_kernel(QuantizeArgs a) {
  const int p = blockIdx.x, b = blockIdx.y;
  const int L = a.seq_lens[b];
  const int P = a.src.page_size;
  if ((int64_t)p * P >= L) return;
  const int32_t pg_in = page_of(a.src, b, p), pg_out = page_of(a.dst, b, p);
  if (pg_in < 0 || pg_out < 0) return;
  const int valid = min(P, L - p * P);
  const int gc = a.src.groups;
  const char* in = (const char*)a.src.pool + (int64_t)pg_in * P * (2 * gc * DH + DR) * 2;
  char* out = (char*)a.dst.pool + (int64_t)pg_out * P * (2 * gc * DH + 2 * DR);
  // K plane: output vector (j, 2 kp + h, slot) <- input vectors (j, 4 kp + h, slot) and (j, 4 kp + 2 + h, slot)
  const int nk = gc * (DH / 16) * P;
  for (int idx = threadIdx.x; idx < nk; idx += 256) {
    const int slot = idx % P, v = (idx / P) % (DH / 16), j = idx / (P * (DH / 16));
    if (slot >= valid) continue;
    const int kp = v >> 1, h = v & 1;
    const char* src = in + ((int64_t)(j * (DH / 8) + 4 * kp + h) * P + slot) * 16;
    const u32x2 lo = e4m3x8(*(const u32x4*)src, a.k_inv_scale);
    const u32x2 hi = e4m3x8(*(const u32x4*)(src + (int64_t)2 * P * 16), a.k_inv_scale);
    *(u32x4*)(out + (int64_t)idx * 16) = u32x4{lo[0], lo[1], hi[0], hi[1]};
  }
  // V plane: output vector (j, T, d, h): tokens 32 T + 8 h + i (bytes 0..7) and 32 T + 16 + 8 h + i (bytes 8..15)
  //          <- input vectors (j, token block 4 T + h, d) and (j, token block 4 T + 2 + h, d)
  const int nv = gc * (P / 32) * DH * 2;
  const char* vin = in + (int64_t)gc * P * DH * 2;
  char* vout = out + (int64_t)gc * P * DH;
  for (int idx = threadIdx.x; idx < nv; idx += 256) {
    const int h = idx & 1, d = (idx >> 1) % DH, T = (idx >> 1) / DH % (P / 32), j = (idx >> 1) / (DH * (P / 32));
    const int t0 = 32 * T + 8 * h;  // first token of bytes 0..7; bytes 8..15 start 16 tokens further
    if (t0 >= valid) continue;
    const u32x2 lo = e4m3x8(*(const u32x4*)(vin + ((int64_t)(j * (P / 8) + 4 * T + h) * DH + d) * 16), a.v_inv_scale);
    const u32x2 hi = e4m3x8(*(const u32x4*)(vin + ((int64_t)(j * (P / 8) + 4 * T + 2 + h) * DH + d) * 16), a.v_inv_scale);
    u32x4 o = {lo[0], lo[1], hi[0], hi[1]};
    u32x4* dst = (u32x4*)(vout + (int64_t)idx * 16);
    if (t0 + 24 <= valid) {
      *dst = o;  // all 16 tokens of the vector exist
    } else {     // the sequence ends inside the vector: keep the bytes of the tokens that do not exist
      const u32x4 old = *dst;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        uint32_t keep = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int tok = t0 + 16 * (w >> 1) + 4 * (w & 1) + k;
          if (tok >= valid) keep |= 0xffu << (8 * k);
        }
        o[w] = (o[w] & ~keep) | (old[w] & keep);
      }
      *dst = o;
    }
  }
  // k_R plane: 16-bit vectors copied as they are
  const int nr = (DR / 8) * P;
  const char* rin = in + (int64_t)2 * gc * P * DH * 2;
  char* rout = out + (int64_t)2 * gc * P * DH;
  for (int idx = threadIdx.x; idx < nr; idx += 256)
    if (idx % P < valid) *(u32x4*)(rout + (int64_t)idx * 16) = *(const u32x4*)(rin + (int64_t)idx * 16);
}

// Cache switch 16-bit latent cache -> 8-bit latent cache of the absorb path (gqla.h: code rows [P][r_kv], then k_R
// [P][d_r] in 16 bits).  One workgroup per (logical page, sequence); a lane converts 8 latent elements at a time, so a
// wave reads and writes whole rows; only tokens t < L_b are touched.
template <int RKV, int DR>
__global__ void __launch_bounds__(256) quantize_latent_kernel(QuantizeArgs a) {
  const int p = blockIdx.x, b = blockIdx.y;
  const int L = a.seq_lens[b];
  const int P = a.src.page_size;
  if ((int64_t)p * P >= L) return;
  const int32_t pg_in = page_of(a.src, b, p), pg_out = page_of(a.dst, b, p);
  if (pg_in < 0 || pg_out < 0) return;
  const int valid = min(P, L - p * P);
  const char* in = (const char*)a.src.pool + (int64_t)pg_in * P * (RKV + DR) * 2;
  char* out = (char*)a.dst.pool + (int64_t)pg_out * P * (RKV + 2 * DR);
  constexpr int VC = RKV / 8, VR = DR / 8;  // 16-byte input vectors per row: latent, RoPE key
  for (int idx = threadIdx.x; idx < valid * VC; idx += 256) {
    const int slot = idx / VC, v = idx % VC;
    const u32x2 c = e4m3x8(*(const u32x4*)(in + ((int64_t)slot * (RKV + DR) + v * 8) * 2), a.k_inv_scale);
    *(u32x2*)(out + (int64_t)slot * RKV + v * 8) = c;
  }
  for (int idx = threadIdx.x; idx < valid * VR; idx += 256) {
    const int slot = idx / VR, v = idx % VR;
    *(u32x4*)(out + (int64_t)P * RKV + ((int64_t)slot * DR + v * 8) * 2) =
        *(const u32x4*)(in + ((int64_t)slot * (RKV + DR) + RKV + v * 8) * 2);
  }
}

}  // namespace

hipError_t launch_quantize_latent(const QuantizeArgs& a, hipStream_t s) {
  quantize_latent_kernel<512, 64><<<dim3(a.src.max_pages, a.B), 256, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_quantize_expanded(const QuantizeArgs& a, hipStream_t s) {
  quantize_expanded_kernel<128, 64><<<dim3(a.src.max_pages, a.B), 256, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace gqla
