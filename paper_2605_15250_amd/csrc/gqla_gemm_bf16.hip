// The two dense contractions around the decode kernels, bf16 MFMA with fp32 accumulation:
//   query absorption  q_hat = W_UK[j] q_C              (paper Sec. 3.1, MQA-absorb equation, line 1)
//   cache expansion   K_C = W_UK^T c,  V = W_UV^T c    (Sec. 3.1, "Two equivalent decoding paths": one-shot expand)
#include "gqla_device.h"
#include "gqla_lds.h"

namespace gqla {

namespace {

// ---- query absorption ------------------------------------------------------------------------------------
// One wave per (group j, 32 query rows of the group, 128 latent dims):
//   Qhat^T[r][row] = W_UK[j][r][d] * Q_C^T[d][row]   A = weight rows straight from global (d contiguous),
//                                                    B = query rows straight from global.
template <int DH, int RKV>
__global__ void __launch_bounds__(256) absorb_query_bf16_kernel(AbsorbQueryArgs a, int rows_per_group) {
  constexpr int KS = DH / 16;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, h = lane >> 5;
  const int j = blockIdx.z;
  const int rblk = blockIdx.y * 4 + wave;  // 128 latent dims each
  if (rblk * 128 >= RKV) return;
  const int x = blockIdx.x * 32 + n;       // x = row * G + head-in-group, row = b * s_q + t
  const bool row_ok = x < rows_per_group;
  const int64_t qrow = row_ok ? (int64_t)(x / a.G) * a.h_q + j * a.G + x % a.G : 0;
  bf16x8 qf[KS];
  const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qf[ks] = row_ok ? *(const bf16x8*)((const __bf16*)a.q_c + qrow * DH + ks * 16 + h * 8) : zero;
  const __bf16* w = (const __bf16*)a.w_uk + ((int64_t)j * RKV + rblk * 128 + n) * DH + h * 8;
  f32x16 acc[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[mt][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      acc[mt] = mfma32(*(const bf16x8*)(w + (int64_t)mt * 32 * DH + ks * 16), qf[ks], acc[mt]);
  }
  if (!row_ok) return;
  __bf16* out = (__bf16*)a.q_hat + qrow * RKV + rblk * 128;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      u32x2 v = {pack_bf16(acc[mt][4 * q], acc[mt][4 * q + 1]), pack_bf16(acc[mt][4 * q + 2], acc[mt][4 * q + 3])};
      *(u32x2*)(out + mt * 32 + 8 * q + 4 * h) = v;
    }
}

// ---- cache expansion -----------------------------------------------------------------------------------------
// One workgroup of 8 waves per (256-token block, sequence); wave w owns 32 tokens.  Each wave keeps its tokens'
// latent rows as 32 register fragments (lane = token, 8 consecutive latent dims per k-step) and reuses them for
// every group and for both K and V, so the latent is read from HBM once.  The weight matrix of one (group, kind)
// at a time ([r_kv][d_h], 128 KB) is staged in LDS and read transposed:
//   K^T[d][tok] = W_UK^T[d][r] * C^T[r][tok]     A = weight fragment, B = latent fragment
//   V[tok][d]   = C[tok][r]    * W_UV[r][d]      A = latent fragment, B = weight fragment (same register contents)
// The two output orientations put 4 consecutive dims (K plane) or 4 consecutive tokens (V plane) of the expanded
// page's 8-element vectors in one lane.
template <int DH, int RKV, int DR>
__global__ void __launch_bounds__(512) expand_bf16_kernel(ExpandArgs a) {
  constexpr int W = RKV + DR;
  constexpr int KS = RKV / 16;
  constexpr int MT = DH / 32;
  static_assert(MT % 2 == 0, "output tiles are processed in pairs that share a 64-column panel");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 31, h = lane >> 5;
  const int b = blockIdx.y;
  const int L = a.seq_lens[b];
  const int tok0 = blockIdx.x * 256;
  if (tok0 >= L) return;  // whole workgroup
  const int P = a.latent.page_size;
  const int gc = a.group_count;
  const int tokw = tok0 + wave * 32;  // first token of this wave (a wave never straddles a page: P % 32 == 0)
  int32_t pg_in = -1, pg_out = -1;
  if (tokw < L) {
    pg_in = page_of(a.latent, b, tokw / P);
    pg_out = page_of(a.expanded, b, tokw / P);
  }
  const bool wave_ok = pg_in >= 0 && pg_out >= 0;  // wave-uniform
  const int slot0 = tokw % P;
  const bool tok_ok = wave_ok && (tokw + n < L);

  // latent rows of this wave's 32 tokens as fragments (lane = token, 8 consecutive latent dims per k-step); rows past
  // L_b are read from a clamped address and zeroed (their products are never stored)
  bf16x8 xf[KS];
  const int n_ld = tok_ok ? n : 0;
  const __bf16* in_row = (const __bf16*)a.latent.pool + ((int64_t)(wave_ok ? pg_in : 0) * P + slot0 + n_ld) * W;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    xf[ks] = *(const bf16x8*)(in_row + ks * 16 + h * 8);
    if (!tok_ok) xf[ks] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
  }

  __bf16* out_page = (__bf16*)a.expanded.pool + (int64_t)(wave_ok ? pg_out : 0) * P * (2 * gc * DH + DR);
  // k_R plane: a straight copy, 8 dims (16 bytes) per lane and step
  if (tok_ok) {
#pragma unroll
    for (int cb = h; cb < DR / 8; cb += 2) {
      const u32x4 v = *(const u32x4*)(in_row + RKV + cb * 8);
      *(u32x4*)(out_page + (int64_t)2 * gc * DH * P + ((int64_t)cb * P + slot0 + n) * 8) = v;
    }
  }

  const TrNatural tr = make_tr_natural(lane);
  for (int jj = 0; jj < gc; ++jj) {
#pragma unroll 1
    for (int kind = 0; kind < 2; ++kind) {
      __syncthreads();  // previous weight matrix no longer read
      const char* wsrc = (const char*)(kind ? a.w_uv : a.w_uk) + (int64_t)(a.group_begin + jj) * RKV * DH * 2;
      stage_panels_full<RKV, DH / 64, 8, DH * 2>(smem, wsrc, wave, lane);
      wait_all_memory();
      __syncthreads();
      if (!wave_ok) continue;
#pragma unroll 1
      for (int mtp = 0; mtp < MT / 2; ++mtp) {  // output tiles 2*mtp, 2*mtp + 1: both in panel mtp
        const char* panel = smem + mtp * (RKV * 128);
        f32x16 acc0, acc1;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc0[i] = acc1[i] = 0.f;
        bf16x8 w0 = tr_natural_frag<RKV>(panel, tr, 0, 0), w1 = tr_natural_frag<RKV>(panel, tr, 0, 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 c0 = w0, c1 = w1;
          if (ks + 1 < KS) {
            w0 = tr_natural_frag<RKV>(panel, tr, ks + 1, 0);
            w1 = tr_natural_frag<RKV>(panel, tr, ks + 1, 1);
          }
          if (kind == 0) {  // K^T[d][tok] = W_UK^T[d][r] * C^T[r][tok]
            acc0 = mfma32(c0, xf[ks], acc0);
            acc1 = mfma32(c1, xf[ks], acc1);
          } else {          // V[tok][d] = C[tok][r] * W_UV[r][d]
            acc0 = mfma32(xf[ks], c0, acc0);
            acc1 = mfma32(xf[ks], c1, acc1);
          }
        }
        if (kind == 0) {
          // lane = token n, registers = dims 32*mt + 8*q + 4*h + 0..3  ->  half of one 8-dim vector of the K plane
          if (tok_ok) {
            __bf16* kb = out_page + (int64_t)jj * DH * P + (int64_t)(slot0 + n) * 8 + 4 * h;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              u32x2 v0 = {pack_bf16(acc0[4 * q], acc0[4 * q + 1]), pack_bf16(acc0[4 * q + 2], acc0[4 * q + 3])};
              u32x2 v1 = {pack_bf16(acc1[4 * q], acc1[4 * q + 1]), pack_bf16(acc1[4 * q + 2], acc1[4 * q + 3])};
              *(u32x2*)(kb + (int64_t)(8 * mtp + q) * P * 8) = v0;
              *(u32x2*)(kb + (int64_t)(8 * mtp + 4 + q) * P * 8) = v1;
            }
          }
        } else {
          // lane = dim 32*mt + n, registers = tokens tokw + 8*q + 4*h + 0..3  ->  half of one 8-token vector of the V plane
          __bf16* vb = out_page + (int64_t)gc * DH * P + (int64_t)jj * DH * P;
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const f32x16& acc = half ? acc1 : acc0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int tk = tokw + 8 * q + 4 * h;  // first of 4 tokens
              __bf16* dst = vb + ((int64_t)((slot0 >> 3) + q) * DH + (2 * mtp + half) * 32 + n) * 8 + 4 * h;
              if (tk + 3 < L) {
                u32x2 v = {pack_bf16(acc[4 * q], acc[4 * q + 1]), pack_bf16(acc[4 * q + 2], acc[4 * q + 3])};
                *(u32x2*)dst = v;
              } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                  if (tk + e < L) dst[e] = (__bf16)acc[4 * q + e];
              }
            }
          }
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_absorb_query_bf16(const AbsorbQueryArgs& a, hipStream_t s) {
  const int rows_per_group = a.rows * a.G;
  dim3 grid((rows_per_group + 31) / 32, (512 / 128 + 3) / 4, a.g);
  absorb_query_bf16_kernel<128, 512><<<grid, 256, 0, s>>>(a, rows_per_group);
  return hipGetLastError();
}

hipError_t launch_expand_bf16(const ExpandArgs& a, hipStream_t s) {
  constexpr int kLds = 512 * 128 * 2;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)expand_bf16_kernel<128, 512, 64>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int64_t max_tokens = (int64_t)a.latent.max_pages * a.latent.page_size;
  dim3 grid((unsigned)((max_tokens + 255) / 256), a.B);
  expand_bf16_kernel<128, 512, 64><<<grid, 512, kLds, s>>>(a);
  return hipGetLastError();
}

}  // namespace gqla
