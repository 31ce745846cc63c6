// The steps either side of the decode path: the decoupled rotary embedding of the step's q^R and k^R (Sec. 3.1,
// "Architecture") and the output projection y = W^O [o_1; ...; o_hq] (last line of both path equations).
#include <type_traits>

#include "gqla_device.h"

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
// waves owns 128 output columns x up to 128 rows x a range of k; wave w owns 32 of the columns, whose rows of W^O it
// reads straight from global memory as MFMA A operands (64 contiguous bytes per lane and 64-element block: inside a
// block lane (n, h) holds k = 32 h + 8 v .. + 7 at its v-th k-step, and the B operand uses the same assignment); the
// rows of o, shared by the four waves, go through LDS as planes of 8-element vectors.  All loads of a 256-element phase
// are issued at once.  With more than one k-range the fp32 partial sums go to the caller's scratch and a second kernel
// adds them in a fixed order.
constexpr int kOpN = 128, kOpM = 128, kOpK = 256;
constexpr int kOpPlane = kOpM + 1;                   // plane stride in 16-byte vectors (odd: writes of a row spread over banks)
constexpr int kOpLds = (kOpK / 8) * kOpPlane * 16;

// MT: 32-row tiles per row block (2 when the call has at most 64 rows, else 4).  PIPE: the loads of the next phase are
// issued before the MFMAs of the current one (two register sets for W^O; affordable with MT = 2).
template <int MT, bool PIPE>
__global__ void __launch_bounds__(256, 2) out_proj_bf16_kernel(OutProjArgs a) {
  constexpr int AI = 4 * MT;                           // staging loads per thread: rows arow + 8 i < 32 MT
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  u32x4* lds = (u32x4*)smem_raw;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, h = lane >> 5;
  const int split = blockIdx.y;
  const int m0 = blockIdx.z * kOpM;
  const int rows = min(32 * MT, a.M - m0);
  const int mts = (rows + 31) / 32;
  const int kbeg = split * a.krange, kend = min(a.K, kbeg + a.krange);
  const int ncol0 = blockIdx.x * kOpN + wave * 32;
  const __bf16* wrow = (const __bf16*)a.w_o + (int64_t)(ncol0 + n) * a.K + 32 * h;
  const int arow = tid >> 5, ac = tid & 31;            // staging role: rows arow + 8 i, vector ac of the phase
  const __bf16* osrc = (const __bf16*)a.o + (int64_t)(m0 + arow) * a.K + ac * 8;

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[mt][i] = 0.f;

  auto load_w = [&](u32x4(&wv)[16], int k0) {
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
      for (int v = 0; v < 4; ++v) wv[blk * 4 + v] = *(const u32x4*)(wrow + k0 + 64 * blk + 8 * v);
  };
  auto load_a = [&](u32x4(&av)[AI], int k0) {
#pragma unroll
    for (int i = 0; i < AI; ++i)
      av[i] = (arow + 8 * i < rows) ? *(const u32x4*)(osrc + (int64_t)8 * i * a.K + k0) : u32x4{0u, 0u, 0u, 0u};
  };
  auto stash = [&](const u32x4(&av)[AI]) {
    __syncthreads();                                   // the previous phase's LDS reads are done
#pragma unroll
    for (int i = 0; i < AI; ++i) lds[ac * kOpPlane + arow + 8 * i] = av[i];
    __syncthreads();
  };
  auto compute = [&](const u32x4(&wv)[16]) {
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const u32x4* plane = lds + (blk * 8 + 4 * h + v) * kOpPlane + n;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          if (mt < mts)
            acc[mt] = mfma32(__builtin_bit_cast(bf16x8, wv[blk * 4 + v]), __builtin_bit_cast(bf16x8, plane[32 * mt]), acc[mt]);
      }
  };

  if constexpr (!PIPE) {
    for (int k0 = kbeg; k0 < kend; k0 += kOpK) {
      u32x4 wv[16], av[AI];
      load_w(wv, k0);
      load_a(av, k0);
      stash(av);
      compute(wv);
    }
  } else {
    u32x4 w0[16], w1[16], av[AI];
    load_w(w0, kbeg);
    load_a(av, kbeg);
    for (int k0 = kbeg; k0 < kend; k0 += 2 * kOpK) {
      stash(av);
      const bool odd = k0 + kOpK < kend;
      if (odd) {
        load_w(w1, k0 + kOpK);
        load_a(av, k0 + kOpK);
      }
      compute(w0);
      if (!odd) break;
      stash(av);
      if (k0 + 2 * kOpK < kend) {
        load_w(w0, k0 + 2 * kOpK);
        load_a(av, k0 + 2 * kOpK);
      }
      compute(w1);
    }
  }

  // C fragment: register 4 q + i holds column ncol0 + 8 q + 4 h + i of row 32 mt + n
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = 32 * mt + n;
    if (m >= rows) continue;
    if (a.ksplit == 1) {
      __bf16* y = (__bf16*)a.y + (int64_t)(m0 + m) * a.D + ncol0 + 4 * h;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *(u32x2*)(y + 8 * q) = u32x2{pack_bf16(acc[mt][4 * q], acc[mt][4 * q + 1]), pack_bf16(acc[mt][4 * q + 2], acc[mt][4 * q + 3])};
    } else {
      float* y = a.partial + ((int64_t)split * a.M + m0 + m) * a.D + ncol0 + 4 * h;
#pragma unroll
      for (int q = 0; q < 4; ++q) *(f32x4*)(y + 8 * q) = f32x4{acc[mt][4 * q], acc[mt][4 * q + 1], acc[mt][4 * q + 2], acc[mt][4 * q + 3]};
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
  for (int k = 1; k < a.ksplit; ++k) s += p[(int64_t)k * total];
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

// k-ranges of the bf16 kernel: as many as keep the launch within two workgroups per compute unit of a 256-unit chip (one
// round of resident workgroups), whole 256-element phases each.  Returns ksplit, sets *krange.
int out_proj_split(int M, int K, int D, int* krange) {
  const int tiles = (D / kOpN) * ((M + kOpM - 1) / kOpM), phases = K / kOpK;
  int want = 512 / tiles;
  if (want > phases) want = phases;
  if (want < 1) want = 1;
  const int per = (phases + want - 1) / want;
  *krange = per * kOpK;
  return (phases + per - 1) / per;
}

hipError_t launch_out_proj_bf16(const OutProjArgs& a, hipStream_t s) {
  static const hipError_t attr2 =
      hipFuncSetAttribute((const void*)out_proj_bf16_kernel<2, true>, hipFuncAttributeMaxDynamicSharedMemorySize, kOpLds);
  static const hipError_t attr4 =
      hipFuncSetAttribute((const void*)out_proj_bf16_kernel<4, false>, hipFuncAttributeMaxDynamicSharedMemorySize, kOpLds);
  if (attr2 != hipSuccess) return attr2;
  if (attr4 != hipSuccess) return attr4;
  const dim3 grid(a.D / kOpN, a.ksplit, (a.M + kOpM - 1) / kOpM);
  if (a.M <= 64) out_proj_bf16_kernel<2, true><<<grid, 256, kOpLds, s>>>(a);
  else out_proj_bf16_kernel<4, false><<<grid, 256, kOpLds, s>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.ksplit == 1) return e;
  const int64_t total = (int64_t)a.M * a.D / 4;
  out_proj_reduce_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace gqla
