// The steps either side of the decode path: the decoupled rotary embedding of the step's q^R and k^R (Sec. 3.1,
// "Architecture") and the output projection y = W^O [o_1; ...; o_hq] (last line of both path equations).
#include <type_traits>

#include "gqla_device.h"
#include "gqla_lds.h"

namespace gqla {

namespace {

// ---- rope_t on the step's rows ------------------------------------------------------------------------------------
// One workgroup per (step token, sequence): position t = L_b - s_q + i; vectors 0 .. h_q-1 are the heads of q^R, vector
// h_q is the k^R part of the token's latent row.  Pair p of a vector turns by t * base^(-2p/d_R); the angle is
// formed and reduced to a fraction of a turn in double (t reaches 10^5 and the fastest pair turns a radian per position);
// sine, cosine and the rotation itself are fp32.
constexpr int kRopeMaxPairs = 256;   // d_R <= 512
template <typename T>
__global__ void __launch_bounds__(512) rope_step_kernel(RopeArgs a) {
  __shared__ float cs_tab[2 * kRopeMaxPairs];
  typedef typename std::conditional<sizeof(T) == 2, uint32_t, f32x2>::type Pair;  // two adjacent elements
  const int i = blockIdx.x, b = blockIdx.y;
  const int half = a.d_r / 2;
  const int vecs = (a.q_r ? a.h_q : 0) + (a.rows ? 1 : 0);
  const int total = vecs * half;
  T* q = a.q_r ? (T*)a.q_r + ((int64_t)b * a.s_q + i) * a.h_q * a.d_r : nullptr;
  T* k = a.rows ? (T*)a.rows + ((int64_t)b * a.s_q + i) * a.row_elems + a.r_kv : nullptr;
  // One pair per thread and pass; four passes are loaded before any is stored, so that a thread pays the memory latency
  // once per four pairs (in place, the stores would otherwise order the loads).  The addresses do not depend on the
  // position: the first four passes are requested before the sequence length is looked at.
  Pair* at[4];
  Pair v[4];
  auto fetch = [&](int base) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int idx = base + j * blockDim.x;
      at[j] = nullptr;
      if (idx < total) {
        const int vec = idx / half;
        T* x = (q && vec < a.h_q) ? q + (int64_t)vec * a.d_r : k;
        at[j] = (Pair*)x + idx % half;
        v[j] = *at[j];
      }
    }
  };
  fetch(threadIdx.x);
  const int t = a.seq_lens[b] - a.s_q + i;
  if (t < 0) return;
  for (int p = threadIdx.x; p < half; p += blockDim.x) {   // one sine / cosine per pair, shared by all vectors of the token
    const double theta = exp2(-2.0 * (double)p / (double)a.d_r * a.log2_base);
    double turns = (double)t * theta * 0.15915494309189535;   // angle / 2 pi; its fraction keeps 1e-11 at t = 10^5
    turns -= floor(turns);
    float sn, cs;
    sincospif(2.0f * (float)turns, &sn, &cs);                  // sin and cos of pi * x: the argument is already reduced
    cs_tab[2 * p] = cs;
    cs_tab[2 * p + 1] = sn;
  }
  __syncthreads();
  for (int base = threadIdx.x; base < total; base += 4 * blockDim.x) {
    if (base != (int)threadIdx.x) fetch(base);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (!at[j]) continue;
      const int p = (base + j * blockDim.x) % half;
      const float c = cs_tab[2 * p], s = cs_tab[2 * p + 1];
      if constexpr (sizeof(T) == 2) {
        const float x0 = bf16_bits_to_float(v[j] & 0xffffu), x1 = bf16_bits_to_float(v[j] >> 16);
        *at[j] = pack_bf16(x0 * c - x1 * s, x0 * s + x1 * c);
      } else {
        *at[j] = f32x2{v[j][0] * c - v[j][1] * s, v[j][0] * s + v[j][1] * c};
      }
    }
  }
}

// ---- output projection, fp32: one thread per output element, k in order ----------------------------------------------
__global__ void __launch_bounds__(64) out_proj_f32_kernel(OutProjArgs a) {
  const int n = blockIdx.x * 64 + threadIdx.x, m = blockIdx.y;
  if (n >= a.D) return;
  const float* o = (const float*)a.o + (int64_t)m * a.K;
  const float* w = (const float*)a.w_o + (int64_t)n * a.K;
  float acc = 0.f;
  for (int k = 0; k < a.K; ++k) acc = fmaf(o[k], w[k], acc);
  ((float*)a.y)[(int64_t)m * a.D + n] = acc;
}

// ---- output projection, bf16 ------------------------------------------------------------------------------------------
// Y^T[n][m] = W^O[n][k] o^T[k][m]: few rows (M = B s_q), a weight matrix that is read once from HBM.  A workgroup of 4
// waves owns 128 output columns x up to 128 rows x a range of k.  W^O reaches the matrix cores through LDS: whole
// 128-byte pieces of its rows are requested with LDS-DMA (8 rows x 128 bytes per wave instruction, each lane 16 bytes of
// a row; every byte of every line is fetched exactly once and never passes through registers) into the panel layout of
// gqla_lds.h, in stages of 64 k, and read back as conflict-free 16-byte A fragments.  The rows of o for the stage travel
// the same way and are shared by the waves.  One barrier per stage: stage p is awaited (counted wait: a wave's requests
// complete in order), the barrier makes every wave's share visible and proves that stage p - 1 is no longer read, whose
// buffer then takes the requests of stage p + 3.  With more than one k-range the fp32 partial sums go to the caller's
// scratch and a second kernel adds them in a fixed order.
// What bounds it (measured, K = 16384, D = 7168, 224 workgroups): 8 rows stream W^O at 6.7 TB/s; the rows of o come out of
// L2 once per column tile, as many bytes as W^O itself at 128 rows, and cost 0.1 us per stage and 8 KB there.
constexpr int kOpN = 128;                    // output columns per workgroup
constexpr int kOpK = 256;                    // granule of the k-ranges
constexpr int kOsK = 64;                     // k per stage: one 128-byte panel per row
constexpr int kOsStages = 4;                 // ring depth (measured: five and six stages, which would still fit, change nothing)
constexpr int kOsWBytes = kOpN * 128;        // W^O part of a stage: 128 rows (output columns) x 128 bytes
template <int MT>
constexpr int out_proj_lds() { return kOsStages * (kOsWBytes + 32 * MT * 128); }

template <int MT>
__global__ void __launch_bounds__(256) out_proj_bf16_kernel(OutProjArgs a) {
  constexpr int OB = 32 * MT * 128;          // o part of a stage: 32 MT rows x 128 bytes
  constexpr int STAGE = kOsWBytes + OB;
  constexpr int NS = kOsStages;
  constexpr int PER = 4 + MT;                // LDS-DMA requests per wave and stage: 16 + 4 MT blocks of 8 rows over 4 waves
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 31, h = lane >> 5;
  // Work item of this workgroup.  Workgroups are dealt to the chip's eight dies in turn (die = id mod 8), each die with an
  // L2 of its own, while items are numbered k-range first, then column tile, then row block: die e takes a contiguous run
  // of items, so that the workgroups of a die share one or two k-ranges of o (which then stay in that L2 while W^O streams
  // through it) and the row blocks that read the same piece of W^O sit side by side.
  const int ncol = a.D / kOpN, nz = (a.M + 32 * MT - 1) / (32 * MT);
  const int total = ncol * nz * a.ksplit;
  const int die = blockIdx.x & 7, per_die = total >> 3, extra = total & 7;
  const int item = die * per_die + min(die, extra) + (blockIdx.x >> 3);
  const int split = item / (ncol * nz);
  const int col_tile = (item / nz) % ncol;
  const int m0 = (item % nz) * 32 * MT;
  const int rows = min(32 * MT, a.M - m0);
  const int kbeg = split * a.krange, kend = min(a.K, kbeg + a.krange);
  const int nst = (kend - kbeg) / kOsK;
  const int col0 = col_tile * kOpN;
  const int64_t stride = (int64_t)a.K * 2;   // bytes from one row of W^O (or of o) to the next

  // staging role of this lane inside a block of 8 rows: row (lane >> 3) of the block, and the 16-byte chunk of the row
  // that the panel layout wants at LDS position lane & 7 (blocks of one wave are 4 apart, so the swizzle term is fixed)
  const int srow = lane >> 3;
  const int schunk = (lane & 7) ^ ((4 * wave + (lane >> 4)) & 7);
  const uint32_t w_off = (uint32_t)(srow * stride + schunk * 16);
  const char* wsrc = (const char*)a.w_o + (int64_t)col0 * stride + (int64_t)kbeg * 2;
  const char* osrc = (const char*)a.o + (int64_t)m0 * stride + (int64_t)kbeg * 2;
  // rows of o beyond the call's last row read that last row instead (their results are never stored)
  uint32_t o_off[MT];
#pragma unroll
  for (int j = 0; j < MT; ++j) o_off[j] = (uint32_t)(min(8 * (wave + 4 * j) + srow, rows - 1) * stride + schunk * 16);

  // The stages of a k-range are taken in rotated order, from a start that differs from one column tile to the next:
  // rows of W^O lie a multiple of 512 bytes apart, so workgroups that walk their k-ranges in step would ask the same
  // few memory channels for everything at any one moment.
  int kpos = (int)((col_tile * 9u) % (unsigned)max(nst, 1));
  int fill = 0;                 // ring slot of the next request
  auto request = [&]() {        // this wave's share of the next stage
    char* buf = smem + fill * STAGE;
    fill = fill + 1 == NS ? 0 : fill + 1;
    const char* wk = wsrc + (int64_t)kpos * (kOsK * 2);
    const char* ok = osrc + (int64_t)kpos * (kOsK * 2);
    kpos = kpos + 1 == nst ? 0 : kpos + 1;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int blk = wave + 4 * j;
      const uint32_t dst = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t)(buf + blk * 1024));
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" : : "s"(dst), "v"(w_off), "s"(wk + (int64_t)blk * 8 * stride) : "memory");
    }
#pragma unroll
    for (int j = 0; j < MT; ++j) {
      const int blk = wave + 4 * j;
      const uint32_t dst = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t)(buf + kOsWBytes + blk * 1024));
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(dst), "v"(o_off[j]), "s"(ok) : "memory");
    }
  };

  // Output tile of a wave: CW x RW blocks of 32 columns x 32 rows (64 rows: the four waves side by side, 1 x 2 each;
  // 128 rows: two by two waves, 2 x 2 each, so that a fragment read from LDS serves two matrix instructions).
  constexpr int CW = MT / 2, RW = 2, NWC = kOpN / (32 * CW);
  const int wc = wave % NWC, wr = wave / NWC;
  f32x16 acc[CW][RW];
#pragma unroll
  for (int c = 0; c < CW; ++c)
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[c][r][i] = 0.f;
  struct Frags {
    bf16x8 w[CW], o[RW];
  };
  auto load_frags = [&](Frags& f, const char* wb, int ks) {
#pragma unroll
    for (int c = 0; c < CW; ++c) f.w[c] = row_frag<kOpN>(wb, 32 * (CW * wc + c) + n, 2 * ks + h);
#pragma unroll
    for (int r = 0; r < RW; ++r) f.o[r] = row_frag<32 * MT>(wb + kOsWBytes, 32 * (RW * wr + r) + n, 2 * ks + h);
  };
  auto multiply = [&](const Frags& f) {
#pragma unroll
    for (int c = 0; c < CW; ++c)
#pragma unroll
      for (int r = 0; r < RW; ++r) acc[c][r] = mfma32(f.w[c], f.o[r], acc[c][r]);
  };

#pragma unroll
  for (int st = 0; st < NS - 1; ++st)
    if (st < nst) request();
  int slot = 0;                 // ring slot of the stage being multiplied
  for (int st = 0; st < nst; ++st) {
    // stage st has landed when at most the requests of the stages behind it (up to NS - 2 of them) are outstanding
    const int behind = min(nst - 1 - st, NS - 2);
    static_for<NS - 1>([&](auto b) {
      if (behind == decltype(b)::value) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(decltype(b)::value * PER) : "memory");
    });
    __syncthreads();
    if (st + NS - 1 < nst) request();
    // fragments are read two k-steps ahead of the matrix instructions that use them: only the first read of a stage is
    // waited for with nothing else to do (one wave per SIMD: no other wave would fill the gap)
    const char* wb = smem + slot * STAGE;
    slot = slot + 1 == NS ? 0 : slot + 1;
    Frags fa, fb;
    load_frags(fa, wb, 0);
    load_frags(fb, wb, 1);
    __builtin_amdgcn_sched_barrier(0);
    multiply(fa);
    load_frags(fa, wb, 2);
    __builtin_amdgcn_sched_barrier(0);
    multiply(fb);
    load_frags(fb, wb, 3);
    __builtin_amdgcn_sched_barrier(0);
    multiply(fa);
    multiply(fb);
  }

  // C fragment: register 4 q + i holds column ncol0 + 8 q + 4 h + i of row n of the block
#pragma unroll
  for (int c = 0; c < CW; ++c) {
    const int ncol0 = col0 + 32 * (CW * wc + c);
#pragma unroll
    for (int r = 0; r < RW; ++r) {
      const int m = 32 * (RW * wr + r) + n;
      if (m >= rows) continue;
      if (a.ksplit == 1) {
        __bf16* y = (__bf16*)a.y + (int64_t)(m0 + m) * a.D + ncol0 + 4 * h;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          *(u32x2*)(y + 8 * q) = u32x2{pack_bf16(acc[c][r][4 * q], acc[c][r][4 * q + 1]), pack_bf16(acc[c][r][4 * q + 2], acc[c][r][4 * q + 3])};
      } else {
        float* y = a.partial + ((int64_t)split * a.M + m0 + m) * a.D + ncol0 + 4 * h;
#pragma unroll
        for (int q = 0; q < 4; ++q) *(f32x4*)(y + 8 * q) = f32x4{acc[c][r][4 * q], acc[c][r][4 * q + 1], acc[c][r][4 * q + 2], acc[c][r][4 * q + 3]};
      }
    }
  }
}

// y = sum over the k-ranges of the fp32 partials, in range order; four columns per thread.
__global__ void __launch_bounds__(256) out_proj_reduce_kernel(OutProjArgs a) {
  const int64_t total = (int64_t)a.M * a.D / 4;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const f32x4* p = (const f32x4*)a.partial + idx;
  f32x4 s = p[0];
  int k = 1;
  for (; k + 3 <= a.ksplit; k += 3) {   // three loads in flight; the sum keeps the range order
    const f32x4 x0 = p[(int64_t)k * total], x1 = p[(int64_t)(k + 1) * total], x2 = p[(int64_t)(k + 2) * total];
    s += x0;
    s += x1;
    s += x2;
  }
  for (; k < a.ksplit; ++k) s += p[(int64_t)k * total];
  *((u32x2*)a.y + idx) = u32x2{pack_bf16(s[0], s[1]), pack_bf16(s[2], s[3])};
}

}  // namespace

hipError_t launch_rope_step(const RopeArgs& a, bool bf16, hipStream_t s) {
  if (bf16) rope_step_kernel<__bf16><<<dim3(a.s_q, a.B), 512, 0, s>>>(a);
  else rope_step_kernel<float><<<dim3(a.s_q, a.B), 512, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_out_proj_f32(const OutProjArgs& a, hipStream_t s) {
  out_proj_f32_kernel<<<dim3((a.D + 63) / 64, a.M), 64, 0, s>>>(a);
  return hipGetLastError();
}

// k-ranges of the bf16 kernel: as many as keep the launch within one workgroup per compute unit of a 256-unit chip (the
// staging ring takes most of a unit's LDS), whole 256-element pieces each.  Returns ksplit, sets *krange.
int out_proj_split(int M, int K, int D, int* krange) {
  const int rows_per_wg = M <= 64 ? 64 : 128;
  const int tiles = (D / kOpN) * ((M + rows_per_wg - 1) / rows_per_wg), phases = K / kOpK;
  int want = 256 / tiles;
  if (want > phases) want = phases;
  if (want < 1) want = 1;
  const int per = (phases + want - 1) / want;
  *krange = per * kOpK;
  return (phases + per - 1) / per;
}

hipError_t launch_out_proj_bf16(const OutProjArgs& a, hipStream_t s) {
  static const hipError_t attr2 = hipFuncSetAttribute((const void*)out_proj_bf16_kernel<2>,
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, out_proj_lds<2>());
  static const hipError_t attr4 = hipFuncSetAttribute((const void*)out_proj_bf16_kernel<4>,
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, out_proj_lds<4>());
  if (attr2 != hipSuccess) return attr2;
  if (attr4 != hipSuccess) return attr4;
  // the kernel's per-lane byte offsets (row inside the tile times the row stride) are 32-bit
  if (a.K > (1 << 24) || a.krange % kOsK) return hipErrorInvalidValue;
  if (a.M <= 64) out_proj_bf16_kernel<2><<<dim3(a.D / kOpN * a.ksplit * ((a.M + 63) / 64)), 256, out_proj_lds<2>(), s>>>(a);
  else out_proj_bf16_kernel<4><<<dim3(a.D / kOpN * a.ksplit * ((a.M + 127) / 128)), 256, out_proj_lds<4>(), s>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.ksplit == 1) return e;
  const int64_t total = (int64_t)a.M * a.D / 4;
  out_proj_reduce_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace gqla
