// fp32 kernels of the GQLA library (vector ALU only, any dims that are multiples of 8).
// They serve the small fp32 configuration; the bf16 MFMA kernels live in their own files.
// One wave (64 lanes) per query row and chunk: lanes run over cached tokens for the logits and over
// output dims for the weighted sum.
#include "gqla_device.h"

namespace gqla {

namespace {

constexpr int kMaxDimsPerLane = 8;  // output dims per lane: d_h <= 512 (GQA), r_kv <= 512 (absorb)

__device__ __forceinline__ float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// q_hat[row, i, r] = sum_d W_UK[j(i)][r][d] * q_c[row, i, d]      (MQA-absorb equation, line 1)
__global__ void absorb_query_f32_kernel(AbsorbQueryArgs a) {
  const int head = blockIdx.x, row = blockIdx.y;
  const int j = head / a.G;
  const float* q = (const float*)a.q_c + ((int64_t)row * a.h_q + head) * a.d_h;
  const float* w = (const float*)a.w_uk + (int64_t)j * a.r_kv * a.d_h;
  float* out = (float*)a.q_hat + ((int64_t)row * a.h_q + head) * a.r_kv;
  for (int r = threadIdx.x; r < a.r_kv; r += blockDim.x) {
    float acc = 0.f;
    for (int d = 0; d < a.d_h; ++d) acc += w[(int64_t)r * a.d_h + d] * q[d];
    out[r] = acc;
  }
}

// Shared body of the two fp32 decode kernels.  kAbsorb: keys = [c | k_R] rows of the latent page, values = c.
// Otherwise: keys = [K_C[j] | k_R], values = V[j] of the expanded page.
template <bool kAbsorb>
__global__ void __launch_bounds__(64) decode_f32_kernel(DecodeArgs a) {
  const int chunk = blockIdx.x, rho = blockIdx.y;  // rho = t * h_q + i
  const int lane = threadIdx.x;
  const ChunkEntry ce = a.chunks[chunk];
  const int t = rho / a.h_q, i = rho % a.h_q, j = i / a.G;
  const int P = a.cache.page_size;
  const int dk = kAbsorb ? a.r_kv : a.d_h;  // content part of the key
  const int dv = kAbsorb ? a.r_kv : a.d_v;  // value dims
  const float* qa = (const float*)a.q_a + ((int64_t)(ce.b * a.s_q + t) * a.h_q + i) * dk;
  const float* qr = (const float*)a.q_r + ((int64_t)(ce.b * a.s_q + t) * a.h_q + i) * a.d_r;
  const float* pool = (const float*)a.cache.pool;
  const int gc = a.cache.groups;
  const int64_t page_elems = kAbsorb ? (int64_t)P * (a.r_kv + a.d_r) : (int64_t)P * (gc * (a.d_h + a.d_v) + a.d_r);
  const int vis_end = min(ce.tok_end, ce.L - a.s_q + t + 1);

  float m_run = GQLA_NEG_INF, l_run = 0.f;
  float o[kMaxDimsPerLane];
  for (int u = 0; u < kMaxDimsPerLane; ++u) o[u] = 0.f;

  for (int tok0 = ce.tok_begin; tok0 < ce.tok_end; tok0 += 64) {
    const int tok = tok0 + lane;
    float z = GQLA_NEG_INF;
    int32_t pg = -1;
    int slot = 0;
    if (tok < vis_end) {
      pg = page_of(a.cache, ce.b, tok / P);
      slot = tok % P;
    }
    if (pg >= 0) {
      const float* base = pool + pg * page_elems;
      float acc = 0.f;
      if (kAbsorb) {
        const float* row = base + (int64_t)slot * (a.r_kv + a.d_r);
        for (int d = 0; d < a.r_kv; ++d) acc += qa[d] * row[d];
        for (int d = 0; d < a.d_r; ++d) acc += qr[d] * row[a.r_kv + d];
      } else {
        for (int d = 0; d < a.d_h; ++d)
          acc += qa[d] * base[((int64_t)(j * (a.d_h / 8) + d / 8) * P + slot) * 8 + d % 8];
        const float* rb = base + (int64_t)gc * P * (a.d_h + a.d_v);
        for (int d = 0; d < a.d_r; ++d) acc += qr[d] * rb[((int64_t)(d / 8) * P + slot) * 8 + d % 8];
      }
      z = acc * a.scale_log2e;
    }
    const float tmax = wave_max(z);
    const float m_new = fmaxf(m_run, tmax);
    const float m_use = (m_new == GQLA_NEG_INF) ? 0.f : m_new;
    const float alpha = fast_exp2(m_run - m_use);
    const float p = (z == GQLA_NEG_INF) ? 0.f : fast_exp2(z - m_use);
    l_run = l_run * alpha + wave_sum(p);
    m_run = m_new;
    for (int u = 0; u < kMaxDimsPerLane; ++u) o[u] *= alpha;
    // weighted sum of values: lane owns dims lane, lane + 64, ...
    for (int src = 0; src < 64; ++src) {
      const float ps = __shfl(p, src);
      const int32_t pgs = __shfl(pg, src);
      const int slots = __shfl(slot, src);
      if (ps == 0.f || pgs < 0) continue;  // wave-uniform
      const float* base = pool + pgs * page_elems;
      for (int u = 0; u < kMaxDimsPerLane; ++u) {
        const int d = lane + 64 * u;
        if (d < dv) {
          float v;
          if (kAbsorb) v = base[(int64_t)slots * (a.r_kv + a.d_r) + d];
          else v = base[(int64_t)gc * P * a.d_h + ((int64_t)(j * (P / 8) + slots / 8) * a.d_v + d) * 8 + slots % 8];
          o[u] += ps * v;
        }
      }
    }
  }
  const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
  float* po = (float*)a.part_o + ((int64_t)chunk * a.M + rho) * dv;
  for (int u = 0; u < kMaxDimsPerLane; ++u) {
    const int d = lane + 64 * u;
    if (d < dv) po[d] = o[u] * inv;
  }
  if (lane == 0) a.part_lse[(int64_t)chunk * a.M + rho] = l_run > 0.f ? (m_run + fast_log2(l_run)) * kLn2 : GQLA_NEG_INF;
}

// Log-sum-exp combine of chunk partials that are already in d_h space.  32 lanes per (b, row), 4 dims per lane and
// step.  One pass over the chunks, kNB at a time so that their loads are in flight together; the running maximum
// moves as in an online softmax (three passes with one dependent load per chunk each would cost three memory
// latencies per chunk).
__global__ void __launch_bounds__(256) combine_kernel(CombineArgs a) {
  constexpr int kNB = 4;
  const int64_t row = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5);  // row = b * M + rho
  if (row >= (int64_t)a.B * a.M) return;
  const int b = (int)(row / a.M), rho = (int)(row % a.M);
  const int s0 = a.first_slot[b], s1 = a.first_slot[b + 1];
  const float* po = (const float*)a.part_o + (int64_t)rho * a.d_h;
  float m = GQLA_NEG_INF, den = 0.f;
  for (int d = (threadIdx.x & 31) * 4; d < a.d_h; d += 128) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    m = GQLA_NEG_INF;
    den = 0.f;
    for (int sb = s0; sb < s1; sb += kNB) {
      float l[kNB];
      f32x4 v[kNB];
#pragma unroll
      for (int k = 0; k < kNB; ++k) {
        const int sc = min(sb + k, s1 - 1);  // clamped: a chunk beyond the range is loaded again and given weight 0
        l[k] = a.part_lse[(int64_t)sc * a.M + rho];
        v[k] = *(const f32x4*)(po + (int64_t)sc * a.M * a.d_h + d);
      }
      float m_new = m;
#pragma unroll
      for (int k = 0; k < kNB; ++k) {
        if (sb + k >= s1) l[k] = GQLA_NEG_INF;
        m_new = fmaxf(m_new, l[k]);
      }
      const float m_use = (m_new == GQLA_NEG_INF) ? 0.f : m_new;
      const float rescale = __expf(m - m_use);  // 0 on the first batch (m = -inf), where den and acc are 0 anyway
      den *= rescale;
      acc *= rescale;
      m = m_new;
#pragma unroll
      for (int k = 0; k < kNB; ++k) {
        const float w = __expf(l[k] - m_use);
        den += w;
        if (w > 0.f) acc += w * v[k];  // a chunk without visible tokens may hold anything
      }
    }
    acc *= 1.f / den;
    *(f32x4*)((float*)a.out + row * a.d_h + d) = acc;
  }
  if (a.lse && (threadIdx.x & 31) == 0) a.lse[row] = m + __logf(den);
}

// fp32 absorb path: combine latent-space partials, then o = W_UV[j]^T o_hat  (MQA-absorb equation, line 6).
__global__ void combine_project_f32_kernel(CombineArgs a) {
  extern __shared__ float o_hat[];  // r_kv floats
  const int rho = blockIdx.x, b = blockIdx.y;
  const int i = rho % a.h_q, j = i / a.G;
  const int s0 = a.first_slot[b], s1 = a.first_slot[b + 1];
  float m = GQLA_NEG_INF;
  for (int s = s0; s < s1; ++s) m = fmaxf(m, a.part_lse[(int64_t)s * a.M + rho]);
  float den = 0.f;
  for (int s = s0; s < s1; ++s) den += __expf(a.part_lse[(int64_t)s * a.M + rho] - m);
  const float* po = (const float*)a.part_o;
  for (int r = threadIdx.x; r < a.r_kv; r += blockDim.x) {
    float acc = 0.f;
    for (int s = s0; s < s1; ++s) {
      const float w = __expf(a.part_lse[(int64_t)s * a.M + rho] - m);
      if (w > 0.f) acc += w * po[((int64_t)s * a.M + rho) * a.r_kv + r];
    }
    o_hat[r] = acc / den;
  }
  __syncthreads();
  const float* w = (const float*)a.w_uv + (int64_t)j * a.r_kv * a.d_h;
  for (int d = threadIdx.x; d < a.d_h; d += blockDim.x) {
    float acc = 0.f;
    for (int r = 0; r < a.r_kv; ++r) acc += w[(int64_t)r * a.d_h + d] * o_hat[r];
    ((float*)a.out)[((int64_t)b * a.M + rho) * a.d_h + d] = acc;
  }
  if (a.lse && threadIdx.x == 0) a.lse[(int64_t)b * a.M + rho] = m + __logf(den);
}

// Cache switch, fp32: one workgroup per (logical page, sequence).
__global__ void expand_f32_kernel(ExpandArgs a) {
  const int p = blockIdx.x, b = blockIdx.y;
  const int L = a.seq_lens[b];
  const int P = a.latent.page_size;
  if ((int64_t)p * P >= L) return;
  const int32_t pg_in = page_of(a.latent, b, p);
  const int32_t pg_out = page_of(a.expanded, b, p);
  if (pg_in < 0 || pg_out < 0) return;
  const int valid = min(P, L - p * P);
  const int W = a.r_kv + a.d_r;
  const int gc = a.group_count;
  const float* in = (const float*)a.latent.pool + (int64_t)pg_in * P * W;
  float* out = (float*)a.expanded.pool + (int64_t)pg_out * P * (gc * (a.d_h + a.d_v) + a.d_r);
  const int nk = gc * a.d_h, per_tok = gc * (a.d_h + a.d_v) + a.d_r;  // K elements, all elements of a token
  for (int idx = threadIdx.x; idx < valid * per_tok; idx += blockDim.x) {
    const int slot = idx / per_tok, e = idx % per_tok;
    const float* c = in + (int64_t)slot * W;
    if (e < per_tok - a.d_r) {
      const int kind = e >= nk;                       // 0: a K_C element, 1: a V element
      const int dim = kind ? a.d_v : a.d_h;           // columns of this kind's weight
      const int x = kind ? e - nk : e, jj = x / dim, d = x % dim;
      const float* w = (const float*)(kind ? a.w_uv : a.w_uk) + (int64_t)(a.group_begin + jj) * a.r_kv * dim;
      float acc = 0.f;
      for (int r = 0; r < a.r_kv; ++r) acc += w[(int64_t)r * dim + d] * c[r];
      if (kind == 0) out[((int64_t)(jj * (a.d_h / 8) + d / 8) * P + slot) * 8 + d % 8] = acc;
      else out[(int64_t)gc * P * a.d_h + ((int64_t)(jj * (P / 8) + slot / 8) * a.d_v + d) * 8 + slot % 8] = acc;
    } else {
      const int d = e - (per_tok - a.d_r);
      out[(int64_t)gc * P * (a.d_h + a.d_v) + ((int64_t)(d / 8) * P + slot) * 8 + d % 8] = c[a.r_kv + d];
    }
  }
}

// Cache switch for the last a.tail positions of every sequence, fp32: one workgroup per (tail token, sequence).
__global__ void expand_tail_f32_kernel(ExpandArgs a) {
  const int t = blockIdx.x, b = blockIdx.y;
  const int L = a.seq_lens[b];
  const int pos = L - a.tail + t;
  if (pos < 0) return;
  const int P = a.latent.page_size;
  const int32_t pg_in = page_of(a.latent, b, pos / P);
  const int32_t pg_out = page_of(a.expanded, b, pos / P);
  if (pg_in < 0 || pg_out < 0) return;
  const int W = a.r_kv + a.d_r;
  const int gc = a.group_count;
  const int slot = pos % P;
  const float* c = (const float*)a.latent.pool + ((int64_t)pg_in * P + slot) * W;
  float* out = (float*)a.expanded.pool + (int64_t)pg_out * P * (gc * (a.d_h + a.d_v) + a.d_r);
  const int nk = gc * a.d_h, per_tok = gc * (a.d_h + a.d_v) + a.d_r;  // K elements, all elements of a token
  for (int e = threadIdx.x; e < per_tok; e += blockDim.x) {
    if (e < per_tok - a.d_r) {
      const int kind = e >= nk;                       // 0: a K_C element, 1: a V element
      const int dim = kind ? a.d_v : a.d_h;           // columns of this kind's weight
      const int x = kind ? e - nk : e, jj = x / dim, d = x % dim;
      const float* w = (const float*)(kind ? a.w_uv : a.w_uk) + (int64_t)(a.group_begin + jj) * a.r_kv * dim;
      float acc = 0.f;
      for (int r = 0; r < a.r_kv; ++r) acc += w[(int64_t)r * dim + d] * c[r];
      if (kind == 0) out[((int64_t)(jj * (a.d_h / 8) + d / 8) * P + slot) * 8 + d % 8] = acc;
      else out[(int64_t)gc * P * a.d_h + ((int64_t)(jj * (P / 8) + slot / 8) * a.d_v + d) * 8 + slot % 8] = acc;
    } else {
      const int d = e - (per_tok - a.d_r);
      out[(int64_t)gc * P * (a.d_h + a.d_v) + ((int64_t)(d / 8) * P + slot) * 8 + d % 8] = c[a.r_kv + d];
    }
  }
}

// Cache compression, fp32: one workgroup per (logical page, sequence); c = A^+ k^C per token, k_R copied.
__global__ void compress_f32_kernel(CompressArgs a) {
  const int p = blockIdx.x, b = blockIdx.y;
  const int L = a.seq_lens[b];
  const int P = a.expanded.page_size;
  if ((int64_t)p * P >= L) return;
  const int32_t pg_in = page_of(a.expanded, b, p), pg_out = page_of(a.latent, b, p);
  if (pg_in < 0 || pg_out < 0) return;
  const int valid = min(P, L - p * P);
  const int g = a.g, W = a.r_kv + a.d_r, K = g * a.d_h;
  const float* in = (const float*)a.expanded.pool + (int64_t)pg_in * P * (g * (a.d_h + a.d_v) + a.d_r);
  float* out = (float*)a.latent.pool + (int64_t)pg_out * P * W;
  for (int idx = threadIdx.x; idx < valid * W; idx += blockDim.x) {
    const int slot = idx / W, e = idx % W;
    float v;
    if (e < a.r_kv) {
      const float* w = (const float*)a.w_inv + (int64_t)e * K;
      float acc = 0.f;
      for (int k = 0; k < K; ++k) {
        const int j = k / a.d_h, d = k % a.d_h;
        acc += w[k] * in[((int64_t)(j * (a.d_h / 8) + d / 8) * P + slot) * 8 + d % 8];
      }
      v = acc;
    } else {
      const int d = e - a.r_kv;
      v = in[(int64_t)g * P * (a.d_h + a.d_v) + ((int64_t)(d / 8) * P + slot) * 8 + d % 8];
    }
    out[(int64_t)slot * W + e] = v;
  }
}

// The step's latent rows into their cache slots (any element type: rows are copied as 16-byte vectors).
// One workgroup per (step token, sequence).
__global__ void append_latent_kernel(AppendArgs a) {
  const int t = blockIdx.x, b = blockIdx.y;
  const int pos = a.seq_lens[b] - a.s_q + t;
  if (pos < 0) return;
  const int P = a.latent.page_size;
  const int32_t pg = page_of(a.latent, b, pos / P);
  if (pg < 0) return;
  const u32x4* src = (const u32x4*)((const char*)a.rows + ((int64_t)b * a.s_q + t) * a.row_bytes);
  u32x4* dst = (u32x4*)((char*)a.latent.pool + ((int64_t)pg * P + pos % P) * a.row_bytes);
  for (int i = threadIdx.x; i < a.row_bytes / 16; i += blockDim.x) dst[i] = src[i];
}

}  // namespace

hipError_t launch_compress_f32(const CompressArgs& a, hipStream_t s) {
  compress_f32_kernel<<<dim3(a.expanded.max_pages, a.B), 256, 0, s>>>(a);
  return hipGetLastError();
}
hipError_t launch_expand_tail_f32(const ExpandArgs& a, hipStream_t s) {
  expand_tail_f32_kernel<<<dim3(a.tail, a.B), 256, 0, s>>>(a);
  return hipGetLastError();
}
hipError_t launch_append_latent(const AppendArgs& a, hipStream_t s) {
  append_latent_kernel<<<dim3(a.s_q, a.B), 128, 0, s>>>(a);
  return hipGetLastError();
}
hipError_t launch_absorb_query_f32(const AbsorbQueryArgs& a, hipStream_t s) {
  absorb_query_f32_kernel<<<dim3(a.h_q, a.rows), 64, 0, s>>>(a);
  return hipGetLastError();
}
hipError_t launch_decode_gqa_f32(const DecodeArgs& a, hipStream_t s) {
  decode_f32_kernel<false><<<dim3(a.n_chunks, a.M), 64, 0, s>>>(a);
  return hipGetLastError();
}
hipError_t launch_decode_absorb_f32(const DecodeArgs& a, hipStream_t s) {
  decode_f32_kernel<true><<<dim3(a.n_chunks, a.M), 64, 0, s>>>(a);
  return hipGetLastError();
}
hipError_t launch_combine_f32(const CombineArgs& a, hipStream_t s) {
  const unsigned blocks = (unsigned)(((int64_t)a.B * a.M + 7) / 8);
  combine_kernel<<<blocks, 256, 0, s>>>(a);
  return hipGetLastError();
}
hipError_t launch_combine_project_f32(const CombineArgs& a, hipStream_t s) {
  combine_project_f32_kernel<<<dim3(a.M, a.B), 128, a.r_kv * sizeof(float), s>>>(a);
  return hipGetLastError();
}
hipError_t launch_expand_f32(const ExpandArgs& a, hipStream_t s) {
  expand_f32_kernel<<<dim3(a.latent.max_pages, a.B), 256, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace gqla
