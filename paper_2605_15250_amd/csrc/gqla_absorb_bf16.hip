// MQA-absorb split-L decode over the latent cache, bf16 MFMA (paper Sec. 3.1, MQA-absorb equation, lines 2-5).
//
// One workgroup of 4 waves per (chunk, block of 128 query rows); wave w owns rows 32w..32w+31 of the block.
// A 64-token latent tile [64][r_kv + d_r] is staged once into LDS (double buffered, global_load_lds) and serves
// every row of the block twice: row-wise as the key operand [c | k_R] and transposed (ds_read_b64_tr_b16) as
// the value operand c:
//   S^T[token][row]  = Kt[token][576] * Qhat^T[576][row]      A = LDS row fragments,   B = queries in registers
//   O^T[r][row]     += C^T[r][token]  * P^T[token][row]       A = LDS transposed frags, B = probabilities
// O^T (512 x 32 fp32 per wave) lives in 256 accumulator registers; the softmax reference maximum is only moved
// (and O^T rescaled) when a row's maximum grows by more than 2^8, so that rescaling is rare.
// Each chunk's normalised latent-space output is written as bf16 with its log-sum-exp; the combine kernel merges
// chunks and applies W_UV.  Intensity h_q s_q (2 r_kv + d_r) / (r_kv + d_r) (Sec. 4.2.1): MFMA-bound for 256 rows.
#include "gqla_device.h"
#include "gqla_lds.h"

namespace gqla {

namespace {

constexpr int kTile = 64;                 // tokens per LDS tile
constexpr int kRowsPerBlock = 128;        // query rows per workgroup
constexpr float kRescaleThreshold = 8.f;  // log2 units

template <int RKV, int DR>
__global__ void __launch_bounds__(256) decode_absorb_bf16_kernel(DecodeArgs a, int row_blocks, int n_chunks_padded) {
  constexpr int W = RKV + DR;        // elements per latent row
  constexpr int RC = W / 8;          // 16-byte chunks per row
  constexpr int KS = W / 16;         // k-steps of the key contraction
  constexpr int DT = RKV / 32;       // 32-wide tiles of the latent output
  constexpr int TILE_BYTES = kTile * W * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  // blockIdx -> (chunk, row block): the row blocks of one chunk get consecutive-by-8 ids so that they run on the
  // same XCD (ids are dealt round-robin over the 8 XCDs) and share the chunk's cache lines in that XCD's L2.
  int chunk, rbk;
  {
    const int id = blockIdx.x;
    const int grp = id / (8 * row_blocks), rem = id % (8 * row_blocks);
    rbk = rem / 8;
    chunk = grp * 8 + rem % 8;
  }
  if (chunk >= a.n_chunks) return;  // whole workgroup leaves together
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, h = lane >> 5;
  const ChunkEntry ce = a.chunks[chunk];

  const int rho = rbk * kRowsPerBlock + wave * 32 + n;  // row = t * h_q + i
  const bool row_ok = rho < a.M;
  const int t = row_ok ? rho / a.h_q : 0;
  const int vis_end = row_ok ? min(ce.tok_end, ce.L - a.s_q + t + 1) : 0;
  const int unmasked_end = min(ce.tok_end, ce.L - a.s_q + 1);
  const bool wave_active = rbk * kRowsPerBlock + wave * 32 < a.M;

  bf16x8 qf[KS];
  {
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    const int64_t qrow = (int64_t)ce.b * a.M + rho;
    const __bf16* ph = (const __bf16*)a.q_a + qrow * RKV + h * 8;
    const __bf16* pr = (const __bf16*)a.q_r + qrow * DR + h * 8;
#pragma unroll
    for (int ks = 0; ks < RKV / 16; ++ks) qf[ks] = row_ok ? *(const bf16x8*)(ph + ks * 16) : zero;
#pragma unroll
    for (int ks = 0; ks < DR / 16; ++ks) qf[RKV / 16 + ks] = row_ok ? *(const bf16x8*)(pr + ks * 16) : zero;
  }

  const int P = a.cache.page_size;
  const char* pool = (const char*)a.cache.pool;
  auto issue_tile = [&](int tok, char* buf) {
    const int32_t pg = page_of(a.cache, ce.b, tok / P);
    const int valid = pg >= 0 ? min(kTile, ce.tok_end - tok) : 0;
    const char* g = pool + ((int64_t)(pg >= 0 ? pg : 0) * P + tok % P) * (W * 2);
    stage_rows<RC>(buf, g, W * 2, kTile, valid, wave, 4, lane);
  };

  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
  float m_ref = GQLA_NEG_INF, l_run = 0.f;

  const int n_tiles = (ce.tok_end - ce.tok_begin + kTile - 1) / kTile;
  issue_tile(ce.tok_begin, smem);
  for (int it = 0; it < n_tiles; ++it) {
    const int tok = ce.tok_begin + it * kTile;
    const char* buf = smem + (it & 1) * TILE_BYTES;
    wait_all_memory();
    __syncthreads();  // tile `it` has landed for every wave; every wave is done reading tile it-1
    if (it + 1 < n_tiles) issue_tile(tok + kTile, smem + ((it + 1) & 1) * TILE_BYTES);

    if (!wave_active) continue;  // waves without query rows only help staging (uniform per wave)
    const bool tile_ok = page_of(a.cache, ce.b, tok / P) >= 0;

    // ---- S^T = Kt * Qhat^T : two 32-token tiles ----
    f32x16 s[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) s[mt][i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) s[mt] = mfma32(row_frag<RC>(buf, 32 * mt + n, 2 * ks + h), qf[ks], s[mt]);
    }

    // ---- online softmax (base 2); register i of s[mt] is token tok + 32*mt + 8*(i/4) + 4*h + i%4 ----
    const bool need_mask = (tok + kTile > unmasked_end) || !row_ok || !tile_ok;
    const int lim = tile_ok ? vis_end : 0;
    float tmax = GQLA_NEG_INF;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        float v = s[mt][i] * a.scale_log2e;
        if (need_mask && tok + 32 * mt + 8 * (i >> 2) + 4 * h + (i & 3) >= lim) v = GQLA_NEG_INF;
        s[mt][i] = v;
        tmax = fmaxf(tmax, v);
      }
    tmax = pair_max(tmax);
    if (__builtin_amdgcn_ballot_w64(tmax > m_ref + kRescaleThreshold) != 0) {
      const float m_new = fmaxf(m_ref, tmax);
      const float alpha = fast_exp2(m_ref - ((m_new == GQLA_NEG_INF) ? 0.f : m_new));
      m_ref = m_new;
      l_run *= alpha;
      if (it > 0) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;
      }
    }
    const float m_use = (m_ref == GQLA_NEG_INF) ? 0.f : m_ref;
    bf16x8 pf[4];  // k-step 2*mt + u: tokens 32*mt + 16*u + {4h..4h+3, 8+4h..8+4h+3}
    float psum = 0.f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        float p[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          p[e] = fast_exp2(s[mt][8 * u + e] - m_use);
          psum += p[e];
        }
        u32x4 w = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
        pf[2 * mt + u] = __builtin_bit_cast(bf16x8, w);
      }
    l_run += psum;

    // ---- O^T += C^T * P^T ----
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int row_a = 16 * kk + 4 * h;  // rows matching elements 0..3 of pf[kk]; elements 4..7 are 8 rows further
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[dt] = mfma32(tr_frag<RC>(buf, row_a, row_a + 8, 32 * dt, lane), pf[kk], o[dt]);
    }
  }

  const float l_tot = pair_sum(l_run);
  if (!row_ok) return;
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  const int64_t prow = (int64_t)chunk * a.M + rho;
  __bf16* po = (__bf16*)a.part_o + prow * RKV;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      u32x2 v = {pack_bf16(o[dt][4 * q] * inv, o[dt][4 * q + 1] * inv), pack_bf16(o[dt][4 * q + 2] * inv, o[dt][4 * q + 3] * inv)};
      *(u32x2*)(po + dt * 32 + 8 * q + 4 * h) = v;
    }
  if (h == 0) a.part_lse[prow] = l_tot > 0.f ? (m_ref + fast_log2(l_tot)) * kLn2 : GQLA_NEG_INF;
}

// ---- combine + latent-output projection: out = W_UV[j]^T (sum_k w_k o_hat_k)   (MQA-absorb equation, line 6) ----
// One workgroup of 4 waves per (group j, 128 query rows of that group); W_UV[j] ([r_kv][d_h], 128 KB) is staged in
// LDS and read transposed: O^T[d][row] = W^T[d][r] * Ohat^T[r][row].
template <int RKV, int DH>
__global__ void __launch_bounds__(256) combine_project_bf16_kernel(CombineArgs a, int rows_per_group) {
  constexpr int RC = DH / 8;
  constexpr int KS = RKV / 16;
  constexpr int MT = DH / 32;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, h = lane >> 5;
  const int j = blockIdx.y;
  stage_rows<RC>(smem, (const char*)a.w_uv + (int64_t)j * RKV * DH * 2, DH * 2, RKV, RKV, wave, 4, lane);

  // row of this lane among the rows of group j: x = (b * s_q + t) * G + head-in-group
  const int x = blockIdx.x * 128 + wave * 32 + n;
  const bool row_ok = x < rows_per_group;
  const int b = row_ok ? x / (a.s_q * a.G) : 0;
  const int t = row_ok ? (x / a.G) % a.s_q : 0;
  const int rho = t * a.h_q + j * a.G + (row_ok ? x % a.G : 0);
  const int s0 = a.first_slot[b], s1 = a.first_slot[b + 1];
  float m = GQLA_NEG_INF;
  for (int s = s0; s < s1; ++s) m = fmaxf(m, a.part_lse[(int64_t)s * a.M + rho]);
  float den = 0.f;
  for (int s = s0; s < s1; ++s) den += __expf(a.part_lse[(int64_t)s * a.M + rho] - m);
  const float inv_den = row_ok ? 1.f / den : 0.f;

  wait_all_memory();
  __syncthreads();

  f32x16 o[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[mt][i] = 0.f;
  const __bf16* po = (const __bf16*)a.part_o;
  for (int ks = 0; ks < KS; ++ks) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (row_ok) {
      for (int s = s0; s < s1; ++s) {
        const float w = __expf(a.part_lse[(int64_t)s * a.M + rho] - m) * inv_den;
        if (w > 0.f) {
          const u32x4 v = *(const u32x4*)(po + ((int64_t)s * a.M + rho) * RKV + ks * 16 + h * 8);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[2 * e] += w * bf16_bits_to_float(v[e] & 0xffffu);
            acc[2 * e + 1] += w * bf16_bits_to_float(v[e] >> 16);
          }
        }
      }
    }
    u32x4 pw = {pack_bf16(acc[0], acc[1]), pack_bf16(acc[2], acc[3]), pack_bf16(acc[4], acc[5]), pack_bf16(acc[6], acc[7])};
    const bf16x8 bfrag = __builtin_bit_cast(bf16x8, pw);
    const int row_a = 16 * ks + 8 * h;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) o[mt] = mfma32(tr_frag<RC>(smem, row_a, row_a + 4, 32 * mt, lane), bfrag, o[mt]);
  }
  if (!row_ok) return;
  __bf16* out = (__bf16*)a.out + ((int64_t)b * a.M + rho) * DH;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      u32x2 v = {pack_bf16(o[mt][4 * q], o[mt][4 * q + 1]), pack_bf16(o[mt][4 * q + 2], o[mt][4 * q + 3])};
      *(u32x2*)(out + mt * 32 + 8 * q + 4 * h) = v;
    }
  if (a.lse && h == 0) a.lse[(int64_t)b * a.M + rho] = m + __logf(den);
}

}  // namespace

hipError_t launch_decode_absorb_bf16(const DecodeArgs& a, hipStream_t s) {
  constexpr int kLds = 2 * kTile * (512 + 64) * 2;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)decode_absorb_bf16_kernel<512, 64>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int row_blocks = (a.M + kRowsPerBlock - 1) / kRowsPerBlock;
  const int chunks_padded = (a.n_chunks + 7) / 8 * 8;
  decode_absorb_bf16_kernel<512, 64><<<chunks_padded * row_blocks, 256, kLds, s>>>(a, row_blocks, chunks_padded);
  return hipGetLastError();
}

hipError_t launch_combine_project_bf16(const CombineArgs& a, hipStream_t s) {
  constexpr int kLds = 512 * 128 * 2;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)combine_project_bf16_kernel<512, 128>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int rows_per_group = a.B * a.s_q * a.G;
  combine_project_bf16_kernel<512, 128><<<dim3((rows_per_group + 127) / 128, a.g), 256, kLds, s>>>(a, rows_per_group);
  return hipGetLastError();
}

}  // namespace gqla
