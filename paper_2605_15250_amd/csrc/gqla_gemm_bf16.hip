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

// The same product for d_h = 128 with both sides of the kernel coalesced (the call is a short kernel in front of every
// absorb decode, and what it costs is how many memory lines its instructions touch): one workgroup per (group j, 32 query
// rows of the group), wave w taking latent dims 128 w .. 128 w + 127.  W_UK[j] (512 rows of 256 bytes, contiguous) is
// staged in LDS with LDS-DMA, 1 KB of consecutive memory per instruction, and read back as conflict-free A fragments; the
// results go back through LDS (a wave's 32 x 128 tile, rows padded to 272 bytes) so that a store instruction writes four
// rows of 256 contiguous bytes instead of 8-byte pieces of 32 rows.  Same MFMAs in the same order as the kernel above.
template <int RKV>
__global__ void __launch_bounds__(256) absorb_query_staged_bf16_kernel(AbsorbQueryArgs a, int rows_per_group) {
  constexpr int DH = 128, KS = DH / 16;
  constexpr int PITCH = 272;                      // bytes per row of the output tile in LDS
  static_assert(RKV == 512, "four waves x 128 latent dims");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ int64_t qrow_of[32];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 31, h = lane >> 5;
  const int j = blockIdx.z;
  stage_panels_full<RKV, DH / 64, 4, DH * 2>(smem, (const char*)a.w_uk + (int64_t)j * RKV * DH * 2, wave, lane);
  const int x = blockIdx.x * 32 + n;       // x = row * G + head-in-group, row = b * s_q + t
  const bool row_ok = x < rows_per_group;
  const int64_t qrow = row_ok ? (int64_t)(x / a.G) * a.h_q + j * a.G + x % a.G : -1;
  if (wave == 0 && h == 0) qrow_of[n] = qrow;
  bf16x8 qf[KS];
  const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qf[ks] = row_ok ? *(const bf16x8*)((const __bf16*)a.q_c + qrow * DH + ks * 16 + h * 8) : zero;
  wait_all_memory();
  __syncthreads();  // W_UK[j] staged
  f32x16 acc[4];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[mt][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) acc[mt] = mfma32(row_frag<RKV>(smem, 128 * wave + 32 * mt + n, 2 * ks + h), qf[ks], acc[mt]);
  }
  __syncthreads();  // every wave is done reading the staged weights: the space becomes the output tiles
  char* tile = smem + wave * (32 * PITCH);
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const u32x2 v = {pack_bf16(acc[mt][4 * q], acc[mt][4 * q + 1]), pack_bf16(acc[mt][4 * q + 2], acc[mt][4 * q + 3])};
      *(u32x2*)(tile + n * PITCH + (mt * 32 + 8 * q + 4 * h) * 2) = v;
    }
  // (only this wave reads its tile: the compiler's wait for the LDS writes is all the ordering needed)
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const int r = 4 * p + (lane >> 4), c = lane & 15;
    const int64_t orow = qrow_of[r];
    const u32x4 v = *(const u32x4*)(tile + r * PITCH + c * 16);
    if (orow >= 0) *(u32x4*)((__bf16*)a.q_hat + orow * RKV + wave * 128 + c * 8) = v;
  }
}

// MFMAs written out so that the latent fragments can live in the accumulation registers (the compiler's own selection
// keeps A and B operands in ordinary registers only): c (+)= A * B with one operand in an AGPR quad.  The *_first forms
// start a sum from zero.  Dependent MFMAs on one accumulator interlock in hardware; before any other instruction reads
// the results, mfma_results_ready() covers the 16-pass latency of the last one.
__device__ __forceinline__ void mfma_va(f32x16& c, bf16x8 a_vgpr, bf16x8 b_agpr) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a_vgpr), "a"(b_agpr));
}
__device__ __forceinline__ void mfma_va_first(f32x16& c, bf16x8 a_vgpr, bf16x8 b_agpr) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(c) : "v"(a_vgpr), "a"(b_agpr));
}
__device__ __forceinline__ void mfma_av(f32x16& c, bf16x8 a_agpr, bf16x8 b_vgpr) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "a"(a_agpr), "v"(b_vgpr));
}
__device__ __forceinline__ void mfma_av_first(f32x16& c, bf16x8 a_agpr, bf16x8 b_vgpr) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(c) : "a"(a_agpr), "v"(b_vgpr));
}
__device__ __forceinline__ void mfma_results_ready(f32x16& c0, f32x16& c1, f32x16& c2, f32x16& c3) {
  asm volatile("s_nop 15\n\ts_nop 7" : "+v"(c0), "+v"(c1), "+v"(c2), "+v"(c3));
}

// ---- cache expansion -----------------------------------------------------------------------------------------
// Step 1 (tiny): the weights of the expanded groups are repacked once per call into MFMA fragment order.  A "stage"
// is one 64-column block of one group's W_UK or W_UV; a group has DH/64 key stages followed by DV/64 value stages
// (DH = DV = 128: two and two; the shape of Sec. 3.2.2, DH = 192 and DV = 256: three and four):
//   packed[jj * (DH + DV)/64 + sub][ks][e][lane][8]  with  lane (m = l % 32, h = l / 32), element i  =
//   W_kind[group_begin + jj][r = 16*ks + 8*h + i][d = 64*mtp + 32*e + m],   (kind, mtp) = stage_kind<DH>(sub)
// i.e. each 1 KB block is one A fragment of W^T (or, with the same register contents, one B fragment of W), and each
// stage is one contiguous 64 KB.
// One workgroup per (stage, 4 k-steps): a [64 latent dims][64 columns] tile of W goes through LDS, read with whole
// 16-byte vectors along the rows and written as whole fragments.
template <int DH, int DV, int RKV>
__global__ void __launch_bounds__(256) pack_weights_bf16_kernel(ExpandArgs a, __bf16* packed) {
  constexpr int KS = RKV / 16;
  constexpr int NSK = DH / 64, NSUB = (DH + DV) / 64;
  __shared__ __attribute__((aligned(16))) __bf16 tile[64][64 + 8];  // rows padded by one vector: column reads spread over the banks
  const int stage = blockIdx.x;  // jj * NSUB + sub
  const int kq = blockIdx.y;     // k-steps 4*kq .. 4*kq + 3
  const int jj = stage / NSUB, sub = stage % NSUB;
  const int kind = sub >= NSK, mtp = kind ? sub - NSK : sub;
  const int dim = kind ? DV : DH;  // columns of this kind's weight
  const __bf16* w = (const __bf16*)(kind ? a.w_uv : a.w_uk) + ((int64_t)(a.group_begin + jj) * RKV + 64 * kq) * dim + 64 * mtp;
  for (int v = threadIdx.x; v < 512; v += 256) {
    const int r = v >> 3, c = (v & 7) * 8;
    *(u32x4*)&tile[r][c] = *(const u32x4*)(w + (int64_t)r * dim + c);
  }
  __syncthreads();
  __bf16* out = packed + (int64_t)stage * KS * 2 * 512 + (int64_t)(4 * kq) * 2 * 512;
  for (int v = threadIdx.x; v < 512; v += 256) {
    const int lane = v & 63, e = (v >> 6) & 1, ksl = v >> 7;
    const int m = lane & 31, h = lane >> 5;
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = tile[16 * ksl + 8 * h + i][32 * e + m];
    *(bf16x8*)(out + (ksl * 2 + e) * 512 + lane * 8) = o;
  }
}

// Step 2: one workgroup of 4 waves per (256-token block, sequence); wave w owns 64 tokens (two 32-token tiles) and,
// alone on its SIMD, the whole 512-entry register file.  Each wave keeps its tokens' latent rows as 2 x 32 register
// fragments (lane = token, 8 consecutive latent dims per k-step) and reuses them for every group and for both K and V,
// so the latent is read from HBM once.  The packed weights stream through LDS one 64 KB stage at a time (LDS-DMA,
// double buffered, the next stage in flight while the current one is multiplied); every weight fragment read from LDS
// feeds two MFMAs (one per token tile):
//   K^T[d][tok] = W_UK^T[d][r] * C^T[r][tok]     A = weight fragment, B = latent fragment
//   V[tok][d]   = C[tok][r]    * W_UV[r][d]      A = latent fragment, B = weight fragment (same register contents)
// The two output orientations put 4 consecutive dims (K plane) or 4 consecutive tokens (V plane) of the expanded
// page's 8-element vectors in one lane.  A stage's results are stored while the next stage is being multiplied, so
// that the end-of-stage wait (which also covers stores on this hardware) finds them long gone.
// With an odd number of stages per group (DH = 192, DV = 256: seven) the two result sets would meet at the group
// boundary, so there the group's last stage stores its results at once instead of in the next stage's shadow.
template <int DH, int DV, int RKV, int DR, bool FP8>
__global__ void __launch_bounds__(256) expand_bf16_kernel(ExpandArgs a, const __bf16* packed) {
  constexpr int W = RKV + DR;
  constexpr int KS = RKV / 16;
  constexpr int STAGE_BYTES = KS * 2 * 1024;  // 64 KB
  constexpr int DEPTH = 2;                    // weight fragments are fetched this many k-steps ahead
  constexpr int NSK = DH / 64, NSUB = (DH + DV) / 64;  // key stages, all stages of a group
  constexpr bool ODD = (NSUB & 1) != 0;
  static_assert(DH % 64 == 0 && DV % 64 == 0, "64-column stages");
  static_assert(!FP8 || (DH == 128 && DV == 128), "the 8-bit page format is written for equal dims of 128");
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
  const int tokw = tok0 + wave * 64;  // first token of this wave (a wave never straddles a page: P % 64 == 0)
  int32_t pg_in = -1, pg_out = -1;
  if (tokw < L) {
    pg_in = page_of(a.latent, b, tokw / P);
    pg_out = page_of(a.expanded, b, tokw / P);
  }
  const bool wave_ok = pg_in >= 0 && pg_out >= 0;  // wave-uniform
  const int slot0 = tokw % P;

  // latent rows of this wave's 64 tokens as fragments, loaded straight into aligned AGPR quads.  Rows past L_b read a
  // clamped (valid) address instead: a token is one MFMA column (K) or row (V), so whatever such a lane computes
  // stays in that token's outputs, and those are never stored.
  bf16x8 xf[2][KS];
  const __bf16* in_page = (const __bf16*)a.latent.pool + (int64_t)(wave_ok ? pg_in : 0) * P * W;
  // FP8: `expanded` is an 8-bit cache (E4M3 code planes and a 16-bit k_R plane, see the header): 2 gc DH + 2 DR bytes per token
  constexpr int EB = FP8 ? 1 : 2;  // bytes per K_C / V element
  char* const page_bytes = (char*)a.expanded.pool + (int64_t)(wave_ok ? pg_out : 0) * P * (gc * (DH + DV) * EB + 2 * DR);
#pragma unroll
  for (int nt = 0; nt < 2; ++nt) {
    const bool tok_ok = wave_ok && (tokw + 32 * nt + n < L);
    const __bf16* in_row = in_page + (int64_t)(slot0 + (tok_ok ? 32 * nt + n : 0)) * W;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(xf[nt][ks]) : "v"(in_row + ks * 16 + h * 8));
    // k_R plane: a straight copy, 8 dims (16 bytes) per lane and step
    if (tok_ok) {
#pragma unroll
      for (int cb = h; cb < DR / 8; cb += 2) {
        const u32x4 v = *(const u32x4*)(in_row + RKV + cb * 8);
        __builtin_nontemporal_store(v, (u32x4*)(page_bytes + (int64_t)gc * (DH + DV) * P * EB + ((int64_t)cb * P + slot0 + 32 * nt + n) * 16));
      }
    }
  }

  // LDS-DMA of one stage: 64 instructions of 1 KB, 16 per wave, linear (the packed layout is already fragment order)
  auto stage_in_step = [&](int stage, char* buf, int u) {  // u = 0..15
    const char* src = (const char*)packed + (int64_t)stage * STAGE_BYTES + wave * (16 * 1024);
    const uint32_t dst = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t)(buf + wave * (16 * 1024)));
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(dst), "v"(lane * 16), "s"(src + u * 1024), "n"(u * 1024) : "memory", "scc");  // the add writes SCC
  };
  auto stage_in = [&](int stage, char* buf) {
#pragma unroll
    for (int u = 0; u < 16; ++u) stage_in_step(stage, buf, u);
  };
  // results of the previous stage ([token tile][32-column half]), kept until the next stage's arithmetic is under way
  f32x16 accs[2][2][2];  // [stage parity][token tile][32-column half]: one set accumulates while the other is stored
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int k = 0; k < 16; ++k) accs[i >> 2][(i >> 1) & 1][i & 1][k] = 0.f;
  // stores address the page through one uniform base and 32-bit offsets (a page is at most a few MB)
  const uint32_t plane_k = (uint32_t)DH * P, plane_v = (uint32_t)DV * P;          // elements of one group's K and V plane
  const uint32_t k_lane = (uint32_t)(slot0 + n) * 8 + (uint32_t)h * P * 8;        // K plane: token slot0 + n, 8-dim block + h
  const uint32_t v_lane = (uint32_t)((slot0 >> 3) + h) * DV * 8 + n * 8;          // V plane: dim n, 8-token block slot0/8 + h
  const bool wave_full = tokw + 64 <= L;                                          // no token of this wave lies beyond L_b
  // One 16-byte store per lane: piece (nt, e, qp) of the previous stage's results; kind, mtp and the piece are compile-time.
  // A lane holds rows 4h..4h+3 of each 8-row block of its column; the two half-waves trade so that lane (n, h) ends up
  // with all 8 rows of block 2*qp + h, i.e. one complete vector of the page layout.
  // 8-bit destination: one 16-byte store per lane and (nt, e): the 32 results of the lane's column as the two code
  // vectors of the page layout (a vector holds 8-row blocks h' and 2 + h' of the 32 rows, each block 4 rows from either
  // half-wave); every result is rounded to bf16 first, so that the codes are those of expanding and then converting.
  auto store_prev8 = [&](int par, int kind, int mtp, int jj, int nt, int e) {
    if (jj < 0 || !wave_ok) return;
    const f32x16& acc = accs[par][nt][e];
    const float inv = kind == 0 ? a.k_inv_scale : a.v_inv_scale;
    uint32_t code[4];  // code[q] = rows 8q + 4h + 0..3
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float x0 = acc[4 * q], x1 = acc[4 * q + 1], x2 = acc[4 * q + 2], x3 = acc[4 * q + 3];
      round_to_bf16x2(x0, x1);
      round_to_bf16x2(x2, x3);
      code[q] = quantize_e4m3x4(x0, x1, x2, x3, inv);
    }
    uint32_t r0, r1, r2, r3;
    half_swap(code[0], code[1], r0, r1);  // lower half: block 0 own, block 0 of the upper half; upper: block 1 of the lower half, block 1 own
    half_swap(code[2], code[3], r2, r3);
    const u32x4 v = {r0, r1, r2, r3};
    if (kind == 0) {
      // lane = token; vector h of pair kp = 2 mtp + e of the K8 plane
      if (wave_full || tokw + 32 * nt + n < L) {
        const uint32_t off = ((uint32_t)(jj * (DH / 16) + 2 * (2 * mtp + e) + h) * P + slot0 + 32 * nt + n) * 16;
        __builtin_nontemporal_store(v, (u32x4*)(page_bytes + off));
      }
    } else {
      // lane = dim 64 mtp + 32 e + n; vector h of 32-token tile (slot0 + 32 nt) / 32 of the V8 plane: tokens 8h + 0..7, 16 + 8h + 0..7
      const uint32_t off = (uint32_t)gc * P * DH +
                           (((uint32_t)(jj * (P / 32) + (slot0 >> 5) + nt) * DH + 64 * mtp + 32 * e + n) * 2 + h) * 16;
      char* dst = page_bytes + off;
      const int tk = tokw + 32 * nt + 8 * h;  // first token of the vector's first half; the second half starts 16 later
      if (wave_full || tk + 23 < L) {
        __builtin_nontemporal_store(v, (u32x4*)dst);
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (tk + 16 * (i >> 3) + (i & 7) < L) dst[i] = (char)((v[i >> 2] >> (8 * (i & 3))) & 0xffu);
      }
    }
  };
  // The two halves of a store are separate so that each fits in the shadow of one matrix instruction: pack_prev rounds
  // and trades (6 vector instructions), emit_prev forms the address and stores.
  auto pack_prev = [&](int par, int nt, int e, int qp) -> u32x4 {
    const f32x16& acc = accs[par][nt][e];
    const int q0 = 2 * qp;
    const uint32_t x0 = pack_bf16(acc[4 * q0], acc[4 * q0 + 1]), x1 = pack_bf16(acc[4 * q0 + 2], acc[4 * q0 + 3]);
    const uint32_t y0 = pack_bf16(acc[4 * q0 + 4], acc[4 * q0 + 5]), y1 = pack_bf16(acc[4 * q0 + 6], acc[4 * q0 + 7]);
    uint32_t r0, r1, r2, r3;
    half_swap(x0, y0, r0, r2);
    half_swap(x1, y1, r1, r3);
    return u32x4{r0, r1, r2, r3};
  };
  auto emit_prev = [&](const u32x4 v, int kind, int mtp, int jj, int nt, int e, int qp) {
    if (jj < 0 || !wave_ok) return;
    const int q0 = 2 * qp;
    if (kind == 0) {
      // lane = token; the vector is dims 64*mtp + 32*e + 8*(2*qp + h) + 0..7 of the K plane
      if (wave_full || tokw + 32 * nt + n < L) {
        const uint32_t off = (uint32_t)jj * plane_k + (uint32_t)(8 * mtp + 4 * e + q0) * P * 8 + 32 * nt * 8 + k_lane;
        __builtin_nontemporal_store(v, (u32x4*)(page_bytes + (size_t)off * 2));
      }
    } else {
      // lane = dim 64*mtp + 32*e + n; the vector is tokens 32*nt + 8*(2*qp + h) + 0..7 of the V plane
      const uint32_t off = (uint32_t)gc * plane_k + (uint32_t)jj * plane_v + (uint32_t)(4 * nt + q0) * DV * 8 + (2 * mtp + e) * 32 * 8 + v_lane;
      __bf16* dst = (__bf16*)(page_bytes + (size_t)off * 2);
      const int tk = tokw + 32 * nt + 8 * (q0 + h);  // first of 8 tokens
      if (wave_full || tk + 7 < L) {
        __builtin_nontemporal_store(v, (u32x4*)dst);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i)
          if (tk + i < L) ((uint16_t*)dst)[i] = (uint16_t)(v[i >> 1] >> (16 * (i & 1)));
      }
    }
  };
  auto store_prev = [&](int par, int kind, int mtp, int jj, int nt, int e, int qp) {
    if (jj < 0 || !wave_ok) return;
    emit_prev(pack_prev(par, nt, e, qp), kind, mtp, jj, nt, e, qp);
  };

  const int n_stages = gc * NSUB;
  stage_in(0, smem);
  wait_all_memory();
  __syncthreads();
  for (int jj = 0; jj < gc; ++jj) {
    static_for<NSUB>([&](auto SUB) __attribute__((always_inline)) {  // compile time: fixes the kind (MFMA operand order) and the result set
      constexpr int sub = decltype(SUB)::value;
      const int stage = jj * NSUB + sub;
      const char* buf = smem + (stage & 1) * STAGE_BYTES + lane * 16;
      f32x16 (&acc)[2][2] = accs[sub & 1];
      // the stage before this one, whose results leave in this stage's shadow (none at the start of a group when the
      // group's last stage has stored its own)
      constexpr int kPrevNone = -1;
      constexpr int psub = sub > 0 ? sub - 1 : (ODD ? kPrevNone : NSUB - 1);
      constexpr int pkind = psub >= NSK, pmtp = pkind ? psub - NSK : psub, ppar = psub & 1;
      const int pjj = psub == kPrevNone ? -1 : (sub == 0 ? jj - 1 : jj);
      if (wave_ok) {
        bf16x8 w[DEPTH + 1][2];
#pragma unroll
        for (int ks = 0; ks < DEPTH; ++ks) {
          w[ks][0] = *(const bf16x8*)(buf + (2 * ks) * 1024);
          w[ks][1] = *(const bf16x8*)(buf + (2 * ks + 1) * 1024);
        }
        // A wave issues in order and is alone on its SIMD: whatever stands between two matrix instructions delays the
        // second one unless it fits into the 32 cycles the first one occupies the pipe.  The other work of a k-step is
        // therefore dealt out one small piece per gap: the two fragment reads for two k-steps ahead, the k-step's share
        // of the next stage's staging, and half of a store of the previous stage's results (pack in the odd k-steps,
        // address and store in the even ones that follow).
        u32x4 packed_piece = {0u, 0u, 0u, 0u};
        auto mm = [&](int ks, int nt, int e) __attribute__((always_inline)) {
          const bf16x8 wf = w[ks % (DEPTH + 1)][e];
          if (sub < NSK) {
            if (ks == 0) mfma_va_first(acc[nt][e], wf, xf[nt][ks]);
            else mfma_va(acc[nt][e], wf, xf[nt][ks]);
          } else {
            if (ks == 0) mfma_av_first(acc[nt][e], xf[nt][ks], wf);
            else mfma_av(acc[nt][e], xf[nt][ks], wf);
          }
          __builtin_amdgcn_sched_barrier(0);
        };
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          __builtin_amdgcn_sched_barrier(0);
          mm(ks, 0, 0);
          if (ks + DEPTH < KS) w[(ks + DEPTH) % (DEPTH + 1)][0] = *(const bf16x8*)(buf + (2 * (ks + DEPTH)) * 1024);
          __builtin_amdgcn_sched_barrier(0);
          mm(ks, 0, 1);
          if (ks + DEPTH < KS) w[(ks + DEPTH) % (DEPTH + 1)][1] = *(const bf16x8*)(buf + (2 * (ks + DEPTH) + 1) * 1024);
          __builtin_amdgcn_sched_barrier(0);
          mm(ks, 1, 0);
          // (after the last stage this stages that stage once more, into the buffer nobody reads any more: no branch)
          if (ks < 16) stage_in_step(min(stage + 1, n_stages - 1), smem + ((stage + 1) & 1) * STAGE_BYTES, ks);
          __builtin_amdgcn_sched_barrier(0);
          mm(ks, 1, 1);
          // the previous stage's results leave in the shadow of this stage's MFMAs
          if constexpr (FP8) {
            if ((ks & 3) == 3 && ks <= 15)  // four pieces (nt, e)
              store_prev8(ppar, pkind, pmtp, pjj, (ks >> 2) >> 1, (ks >> 2) & 1);
          } else if (psub != kPrevNone && ks >= 1 && ks <= 16) {
            const int piece = (ks - 1) >> 1;  // packed at k-step 2 piece + 1, stored at 2 piece + 2
            if (ks & 1) {
              packed_piece = pack_prev(ppar, piece >> 2, (piece >> 1) & 1, piece & 1);  // (before the first stage: zeros, never stored)
            } else {
              emit_prev(packed_piece, pkind, pmtp, pjj, piece >> 2, (piece >> 1) & 1, piece & 1);
            }
          }
        }
        mfma_results_ready(acc[0][0], acc[0][1], acc[1][0], acc[1][1]);
        if constexpr (ODD && !FP8) {
          if (sub == NSUB - 1) {
#pragma unroll
            for (int piece = 0; piece < 8; ++piece) store_prev(sub & 1, 1, sub - NSK, jj, piece >> 2, (piece >> 1) & 1, piece & 1);
          }
        }
      } else {
        stage_in(min(stage + 1, n_stages - 1), smem + ((stage + 1) & 1) * STAGE_BYTES);  // a wave without tokens still stages its share
      }
      wait_all_memory();
      __syncthreads();  // next stage has landed; everyone is done with this stage's buffer
    });
  }
  if constexpr (FP8) {
#pragma unroll
    for (int piece = 0; piece < 4; ++piece) store_prev8((NSUB - 1) & 1, 1, NSUB - 1 - NSK, gc - 1, piece >> 1, piece & 1);
  } else if constexpr (!ODD) {
#pragma unroll
    for (int piece = 0; piece < 8; ++piece) store_prev((NSUB - 1) & 1, 1, NSUB - 1 - NSK, gc - 1, piece >> 2, (piece >> 1) & 1, piece & 1);
  }
}

// ---- cache expansion of the last a.tail positions of every sequence (the step's new tokens) ------------------------
// The B * tail tokens form one list (index = b * tail + t) cut into 32-token tiles; a workgroup is one packed weight
// stage (64 output columns of one group's W_UK or W_UV, see pack_weights_bf16_kernel) times 64 tokens, wave w taking
// the 32-column half w & 1 and the token tile w >> 1:
//   K^T[d][tok] = W_UK^T[d][r] * C^T[r][tok]   and   V^T[d][tok] = W_UV^T[d][r] * C^T[r][tok]
//   A = packed weight fragment straight from global memory (1 KB, contiguous), B = the tokens' latent rows, gathered
//   (lane = token, 8 consecutive latent dims per k-step).
// Tokens of a tile belong to different sequences and pages, so results go out as 8-byte (K plane: 4 consecutive dims
// of one token) and 2-byte (V plane: one token's element of an 8-token vector) stores; with a few hundred tokens per
// step that is a few hundred KB.  The first stage's workgroups also copy the tokens' k_R.
// FP8 = true: `expanded` is an 8-bit cache (E4M3 code planes, see the header); every result is first rounded to bf16,
// the value the 16-bit cache would hold, and then quantised, so that the codes equal those of expanding into a 16-bit
// cache and converting it.
template <int DH, int DV, int RKV, int DR, bool FP8>
__global__ void __launch_bounds__(256) expand_tail_bf16_kernel(ExpandArgs a, const __bf16* packed) {
  constexpr int W = RKV + DR;
  constexpr int KS = RKV / 16;
  constexpr int NSK = DH / 64, NSUB = (DH + DV) / 64;
  static_assert(!FP8 || (DH == 128 && DV == 128), "the 8-bit page format is written for equal dims of 128");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 31, h = lane >> 5;
  const int stage = blockIdx.x;  // jj * NSUB + sub
  const int jj = stage / NSUB, sub = stage % NSUB;
  const int kind = sub >= NSK, mtp = kind ? sub - NSK : sub;
  const int e = wave & 1;
  const int idx = blockIdx.y * 64 + (wave >> 1) * 32 + n;  // this lane's token in the list
  const int P = a.latent.page_size;
  const int gc = a.group_count;
  bool ok = idx < a.B * a.tail;
  int b = 0, pos = 0;
  if (ok) {
    b = idx / a.tail;
    pos = a.seq_lens[b] - a.tail + idx % a.tail;
    ok = pos >= 0;
  }
  int32_t pg_in = -1, pg_out = -1;
  if (ok) {
    pg_in = page_of(a.latent, b, pos / P);
    pg_out = page_of(a.expanded, b, pos / P);
    ok = pg_in >= 0 && pg_out >= 0;
  }
  const int slot = ok ? pos % P : 0;
  // a lane without a token reads row 0 of page 0 (valid memory); its MFMA column is never stored
  const __bf16* row = (const __bf16*)a.latent.pool + ((int64_t)(ok ? pg_in : 0) * P + slot) * W;
  const __bf16* wf = packed + (int64_t)stage * KS * 2 * 512 + e * 512 + lane * 8;
  // Every load of the contraction is in flight before the first MFMA (the call is a chain of short kernels: what it costs
  // is memory latency, paid once this way): the latent fragments go straight into accumulation registers, as in the
  // one-shot kernel, which leaves the ordinary registers to the 32 weight fragments.  One accumulation chain in k order,
  // the one-shot kernel's order: the two produce the same bits.
  bf16x8 xf[KS], wv[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(xf[ks]) : "v"(row + ks * 16 + h * 8));
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) wv[ks] = *(const bf16x8*)(wf + (int64_t)ks * 1024);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  f32x16 acc;
  mfma_va_first(acc, wv[0], xf[0]);
#pragma unroll
  for (int ks = 1; ks < KS; ++ks) mfma_va(acc, wv[ks], xf[ks]);
  asm volatile("s_nop 15\n\ts_nop 7" : "+v"(acc));  // the last MFMA's passes, before anything else reads the results
  if (!ok) return;
  const int d0 = 64 * mtp + 32 * e;  // register i holds dim d0 + 8*(i/4) + 4*h + i%4 of this lane's token
  if constexpr (FP8) {
    char* out8 = (char*)a.expanded.pool + (int64_t)pg_out * P * (2 * gc * DH + 2 * DR);
    const float inv = kind == 0 ? a.k_inv_scale : a.v_inv_scale;
    uint32_t code[4];  // code[q] = dims d0 + 8q + 4h + 0..3
#pragma unroll
    for (int q = 0; q < 4; ++q)
      code[q] = quantize_e4m3x4(round_to_bf16(acc[4 * q]), round_to_bf16(acc[4 * q + 1]), round_to_bf16(acc[4 * q + 2]),
                                round_to_bf16(acc[4 * q + 3]), inv);
    if (kind == 0) {  // dim 32 kp + 16 u + 8 h' + i: here kp = d0/32, u = q/2, h' = q%2, i = 4h + 0..3 -> four consecutive bytes
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *(uint32_t*)(out8 + ((int64_t)(jj * (DH / 16) + 2 * (d0 / 32) + (q & 1)) * P + slot) * 16 + 8 * (q >> 1) + 4 * h) = code[q];
    } else {          // slot 32 T + 16 u + 8 h' + i: one byte per dim
      char* vp = out8 + (int64_t)gc * P * DH + ((int64_t)(jj * (P / 32) + slot / 32) * DH * 2 + ((slot >> 3) & 1)) * 16 +
                 8 * ((slot >> 4) & 1) + (slot & 7);
#pragma unroll
      for (int i = 0; i < 16; ++i)
        vp[(int64_t)(d0 + 8 * (i >> 2) + 4 * h + (i & 3)) * 32] = (char)((code[i >> 2] >> (8 * (i & 3))) & 0xffu);
    }
    if (stage == 0 && e == 0) {
      char* rp = out8 + (int64_t)2 * gc * P * DH;
#pragma unroll
      for (int c = h; c < DR / 8; c += 2) *(u32x4*)(rp + ((int64_t)c * P + slot) * 16) = *(const u32x4*)(row + RKV + c * 8);
    }
    return;
  }
  __bf16* out_page = (__bf16*)a.expanded.pool + (int64_t)pg_out * P * (gc * (DH + DV) + DR);
  if (kind == 0) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const u32x2 v = {pack_bf16(acc[4 * q], acc[4 * q + 1]), pack_bf16(acc[4 * q + 2], acc[4 * q + 3])};
      *(u32x2*)(out_page + ((int64_t)(jj * (DH / 8) + d0 / 8 + q) * P + slot) * 8 + 4 * h) = v;
    }
  } else {
    __bf16* vp = out_page + (int64_t)gc * P * DH + ((int64_t)(jj * (P / 8) + slot / 8) * DV) * 8 + slot % 8;
#pragma unroll
    for (int i = 0; i < 16; ++i) vp[(int64_t)(d0 + 8 * (i >> 2) + 4 * h + (i & 3)) * 8] = (__bf16)acc[i];
  }
  if (stage == 0 && e == 0) {  // k_R of this token: dims 8*c .. 8*c + 7 for c = h, h + 2, ...
    __bf16* rp = out_page + (int64_t)gc * P * (DH + DV);
#pragma unroll
    for (int c = h; c < DR / 8; c += 2) *(u32x4*)(rp + ((int64_t)c * P + slot) * 8) = *(const u32x4*)(row + RKV + c * 8);
  }
}

// ---- cache compression: latent from the expanded keys (Sec. 3.1: the reverse cache switch) --------------------------
// c_s = A^+ k^C_s with the caller's left inverse A^+ ([r_kv][g*d_h], k^C ordered group-major, dim-minor); k_R copied.
// One workgroup of 8 waves per (128 tokens, sequence) computes all r_kv latent dims of its tokens; wave (tw, rw)
// owns tokens [64 tw, 64 tw + 64) x latent dims [128 rw, 128 rw + 128):
//   C^T[r][tok] = A^+[r][k] * K^T[k][tok]
// The contraction runs in stages of 32 k.  Per stage the workgroup stages the [512 x 32] slice of A^+ and the
// [128 tokens x 32] slice of the K_C plane through LDS (registers -> LDS, three buffers, one barrier per stage), as
// planes of 8-element vectors, so that each MFMA operand is one conflict-free 16-byte LDS read; every element of A^+
// is fetched once per 128 tokens instead of once per wave.
constexpr int kCompressKS = 32;                       // contraction elements per stage
constexpr int kCompressTok = 128;                     // tokens per workgroup
template <int RKV>
constexpr int compress_lds_bytes() {
  return 3 * (kCompressKS / 8) * ((RKV + 4) + kCompressTok) * 16;
}

template <int DH, int DV, int RKV, int DR>
__global__ void __launch_bounds__(512) compress_bf16_kernel(CompressArgs a) {
  static_assert(RKV == 512 && DH % kCompressKS == 0, "wave tiling below assumes 4 blocks of 128 latent dims");
  constexpr int NC = kCompressKS / 8;                 // vector planes per stage
  constexpr int WPL = RKV + 4;                        // plane stride of the A^+ tile, in vectors (padding spreads the writes)
  constexpr int BUF = NC * (WPL + kCompressTok);      // vectors per buffer
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  u32x4* smem = (u32x4*)smem_raw;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, h = lane >> 5;
  const int tw = wave & 1, rw = wave >> 1;
  const int b = blockIdx.y;
  const int L = a.seq_lens[b];
  const int tok0 = blockIdx.x * kCompressTok;
  if (tok0 >= L) return;
  const int P = a.expanded.page_size;
  const int g = a.g;
  const int K = g * DH;
  const int64_t in_page_elems = (int64_t)P * (g * (DH + DV) + DR);

  // staging role of this thread: one K vector per stage (token kt of the tile, plane kc) and four A^+ vectors
  const int kt = tid & (kCompressTok - 1), kc = tid >> 7;
  const __bf16* ksrc = nullptr;
  {
    const int tk = tok0 + (kt & 64);
    if (tk < L) {
      const int32_t pg = page_of(a.expanded, b, tk / P);
      if (pg >= 0) ksrc = (const __bf16*)a.expanded.pool + pg * in_page_elems + ((int64_t)kc * P + tk % P + (kt & 63)) * 8;
    }
  }
  const __bf16* wsrc = (const __bf16*)a.w_inv + (int64_t)(tid >> 2) * K + (tid & 3) * 8;   // + i * 128 rows, + stage * 32
  const int wdst = (tid & 3) * WPL + (tid >> 2);                                            // + i * 128
  const int kdst = NC * WPL + kc * kCompressTok + kt;

  // Global memory is read in pairs of stages (64 contraction elements: whole 128-byte lines of A^+, the two halves
  // requested back to back) into two register sets.  Rows of A^+ are 2 g d_h bytes apart, a power of two; as a
  // precaution against all workgroups of an L2 asking for the same address bits at once, every eighth workgroup starts
  // the contraction at a different stage pair and walks it cyclically (measured: neutral on this chip).
  u32x4 wreg[2][4], kreg[2];
  const int stages = K / kCompressKS, pairs = stages / 2;
  const int rot = (int)((blockIdx.x + gridDim.x * blockIdx.y) >> 3) % pairs;
  auto fetch = [&](int e, int step) {                 // half e of the step-th stage pair of this workgroup's walk
    const int pr = step + rot < pairs ? step + rot : step + rot - pairs;
    const int st = 2 * pr + e;
    const int j = st / (DH / kCompressKS), v0 = j * (DH / 8) + (st % (DH / kCompressKS)) * NC;
#pragma unroll
    for (int i = 0; i < 4; ++i) wreg[e][i] = *(const u32x4*)(wsrc + (int64_t)i * 128 * K + st * kCompressKS);
    kreg[e] = ksrc ? *(const u32x4*)(ksrc + (int64_t)v0 * P * 8) : u32x4{0u, 0u, 0u, 0u};
  };
  auto stash = [&](int e, int buf) {
    u32x4* dst = smem + buf * BUF;
#pragma unroll
    for (int i = 0; i < 4; ++i) dst[wdst + i * 128] = wreg[e][i];
    dst[kdst] = kreg[e];
  };

  f32x16 acc[2][4];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt)
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[tt][rt][i] = 0.f;

  auto compute = [&](int buf) {
    const u32x4* wt = smem + buf * BUF;
    const u32x4* ktile = wt + NC * WPL;
#pragma unroll
    for (int ks = 0; ks < kCompressKS / 16; ++ks) {
      u32x4 kf[2], wf[4];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) kf[tt] = ktile[(2 * ks + h) * kCompressTok + 64 * tw + 32 * tt + n];
#pragma unroll
      for (int rt = 0; rt < 4; ++rt) wf[rt] = wt[(2 * ks + h) * WPL + 128 * rw + 32 * rt + n];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
          acc[tt][rt] = mfma32(__builtin_bit_cast(bf16x8, wf[rt]), __builtin_bit_cast(bf16x8, kf[tt]), acc[tt][rt]);
    }
  };

  // Step s (in the rotated order) is computed from buffer s % 3 while step s + 1 goes from registers into buffer
  // (s + 1) % 3 -- last read in iteration s - 2, which every wave has left through the barrier of iteration s - 1.
  // Each register set is refilled from global memory right after it has been written to LDS, two steps before it is
  // needed again.
  fetch(0, 0);
  fetch(1, 0);
  stash(0, 0);
  if (pairs > 1) fetch(0, 1);
  __syncthreads();
  int buf = 0;                                        // buffer of the even step of the pair
  for (int pr = 0; pr < pairs; ++pr) {
    const int b1 = buf == 2 ? 0 : buf + 1, b2 = b1 == 2 ? 0 : b1 + 1;
    stash(1, b1);                                     // odd step of this pair
    if (pr + 1 < pairs) fetch(1, pr + 1);
    compute(buf);
    __syncthreads();
    if (pr + 1 < pairs) stash(0, b2);                 // even step of the next pair
    if (pr + 2 < pairs) fetch(0, pr + 2);
    compute(b1);
    __syncthreads();
    buf = b2;
  }

  const int tokh = tok0 + 64 * tw;                    // this wave's 64 tokens lie in one page
  if (tokh >= L) return;
  const int32_t pg_in = page_of(a.expanded, b, tokh / P), pg_out = page_of(a.latent, b, tokh / P);
  if (pg_in < 0 || pg_out < 0) return;
  const __bf16* in_page = (const __bf16*)a.expanded.pool + pg_in * in_page_elems;
  __bf16* out_page = (__bf16*)a.latent.pool + (int64_t)pg_out * P * (RKV + DR);
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int slot = tokh % P + 32 * tt + n;
    if (tokh + 32 * tt + n >= L) continue;
    __bf16* row = out_page + (int64_t)slot * (RKV + DR);
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const u32x2 v = {pack_bf16(acc[tt][rt][4 * q], acc[tt][rt][4 * q + 1]), pack_bf16(acc[tt][rt][4 * q + 2], acc[tt][rt][4 * q + 3])};
        *(u32x2*)(row + 128 * rw + 32 * rt + 8 * q + 4 * h) = v;
      }
    if (rw == 0) {  // k_R: dims 8c .. 8c + 7 for c = h, h + 2, ...
      const __bf16* rp = in_page + (int64_t)g * P * (DH + DV);
#pragma unroll
      for (int c = h; c < DR / 8; c += 2) *(u32x4*)(row + RKV + c * 8) = *(const u32x4*)(rp + ((int64_t)c * P + slot) * 8);
    }
  }
}

}  // namespace

template <int DH, int DV>
static hipError_t launch_compress_dims(const CompressArgs& a, hipStream_t s) {
  constexpr int lds = compress_lds_bytes<512>();
  static const hipError_t attr =
      hipFuncSetAttribute((const void*)compress_bf16_kernel<DH, DV, 512, 64>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (attr != hipSuccess) return attr;
  const int64_t max_tokens = (int64_t)a.expanded.max_pages * a.expanded.page_size;
  compress_bf16_kernel<DH, DV, 512, 64><<<dim3((unsigned)((max_tokens + kCompressTok - 1) / kCompressTok), a.B), 512, lds, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_compress_bf16(const CompressArgs& a, hipStream_t s) {
  return a.d_h == 192 ? launch_compress_dims<192, 256>(a, s) : launch_compress_dims<128, 128>(a, s);
}

hipError_t launch_absorb_query_bf16(const AbsorbQueryArgs& a, hipStream_t s) {
  const int rows_per_group = a.rows * a.G;
  dim3 grid((rows_per_group + 31) / 32, (512 / 128 + 3) / 4, a.g);
  if (a.d_h == 192) {
    absorb_query_bf16_kernel<192, 512><<<grid, 256, 0, s>>>(a, rows_per_group);
    return hipGetLastError();
  }
  constexpr int kLds = 512 * 128 * 2;   // W_UK[j]
  static const hipError_t attr =
      hipFuncSetAttribute((const void*)absorb_query_staged_bf16_kernel<512>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
  if (attr != hipSuccess) return attr;
  absorb_query_staged_bf16_kernel<512><<<dim3(grid.x, 1, a.g), 256, kLds, s>>>(a, rows_per_group);
  return hipGetLastError();
}

template <int DH, int DV, bool FP8>
static hipError_t launch_expand_tail_dims(const ExpandArgs& a, void* ws, hipStream_t s) {
  constexpr int NSUB = (DH + DV) / 64;
  const int tokens = a.B * a.tail;
  if (a.weights != 2) {
    pack_weights_bf16_kernel<DH, DV, 512><<<dim3(a.group_count * NSUB, 512 / 64), 256, 0, s>>>(a, (__bf16*)ws);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.weights == 1) return e;
  }
  expand_tail_bf16_kernel<DH, DV, 512, 64, FP8><<<dim3(a.group_count * NSUB, (tokens + 63) / 64), 256, 0, s>>>(a, (const __bf16*)ws);
  return hipGetLastError();
}

hipError_t launch_expand_tail_bf16(const ExpandArgs& a, void* ws, hipStream_t s) {
  return a.d_h == 192 ? launch_expand_tail_dims<192, 256, false>(a, ws, s) : launch_expand_tail_dims<128, 128, false>(a, ws, s);
}

hipError_t launch_expand_tail_fp8(const ExpandArgs& a, void* ws, hipStream_t s) { return launch_expand_tail_dims<128, 128, true>(a, ws, s); }

template <int DH, int DV, bool FP8>
static hipError_t launch_expand_one_shot(const ExpandArgs& a, void* ws, hipStream_t s) {
  constexpr int kLds = 2 * (512 / 16) * 2 * 1024;
  constexpr int NSUB = (DH + DV) / 64;
  // once per process (function-local statics are initialised under a lock); an error is reported by every call
  static const hipError_t attr =
      hipFuncSetAttribute((const void*)expand_bf16_kernel<DH, DV, 512, 64, FP8>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
  if (attr != hipSuccess) return attr;
  const int64_t max_tokens = (int64_t)a.latent.max_pages * a.latent.page_size;
  dim3 grid((unsigned)((max_tokens + 255) / 256), a.B);
  pack_weights_bf16_kernel<DH, DV, 512><<<dim3(a.group_count * NSUB, 512 / 64), 256, 0, s>>>(a, (__bf16*)ws);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  expand_bf16_kernel<DH, DV, 512, 64, FP8><<<grid, 256, kLds, s>>>(a, (const __bf16*)ws);
  return hipGetLastError();
}
hipError_t launch_expand_bf16(const ExpandArgs& a, void* ws, hipStream_t s) {
  return a.d_h == 192 ? launch_expand_one_shot<192, 256, false>(a, ws, s) : launch_expand_one_shot<128, 128, false>(a, ws, s);
}
hipError_t launch_expand_fp8(const ExpandArgs& a, void* ws, hipStream_t s) { return launch_expand_one_shot<128, 128, true>(a, ws, s); }

}  // namespace gqla
