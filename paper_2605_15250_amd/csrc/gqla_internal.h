// Internal declarations shared by the host entry points and the HIP kernels of the GQLA library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>

#include "gqla.h"

namespace gqla {

// One row of the chunk table that a decode kernel reads (16 bytes).
struct ChunkEntry {
  int32_t b;          // sequence
  int32_t tok_begin;  // first cached token of the chunk (multiple of page_size)
  int32_t tok_end;    // one past the last token, clipped to L_b
  int32_t L;          // L_b, for the in-step causal mask
};

// Device-side view of a cache pool.
struct CacheView {
  const void* pool;
  const int32_t* page_table;  // may be null: identity map b*max_pages + p
  int32_t page_size, max_pages, num_pages, groups;
};

// Arguments common to both decode kernels.
struct DecodeArgs {
  const void* q_a;  // q_c (GQA path) or q_hat (absorb path)
  const void* q_r;
  CacheView cache;
  const ChunkEntry* chunks;
  int32_t n_chunks;
  void* part_o;      // GQA fp32: fp32 [chunks][M][d_v];  GQA bf16 / 8-bit: fp32 vectors [chunks][M / 32][d_v / 4][32][4] (part_vec_index);  absorb bf16: bf16 vectors [chunks][M / 32][r_kv / 8][32][8] (part_vec_index);  absorb f32: fp32 [chunks][M][r_kv]
  float* part_lse;   // fp32 [chunks][M], natural log
  int32_t B, h_q, g, G, d_h, d_v, r_kv, d_r, s_q, M;  // M = s_q * h_q rows per sequence, row = t*h_q + i; d_v: value dim (GQA path)
  int32_t num_cus;                               // compute units the plan was made for (launch-shape choices only)
  float scale_log2e;                             // softmax scale times log2(e)
};

// Arguments of the combine (and, for the absorb path, combine + W_UV projection) kernels.
struct CombineArgs {
  const void* part_o;
  const float* part_lse;
  const int32_t* first_slot;  // int32[B + 1]
  const void* w_uv;           // absorb path only
  void* out;                  // [B][s_q][h_q][d_h]
  float* lse;                 // optional [B][s_q][h_q]
  int32_t B, h_q, g, G, d_h, r_kv, s_q, M;
};

struct ExpandArgs {
  CacheView latent;
  CacheView expanded;
  const int32_t* seq_lens;
  const void* w_uk;
  const void* w_uv;
  int32_t B, g, d_h, d_v, r_kv, d_r, group_begin, group_count;  // d_h: key dim (columns of W_UK), d_v: value dim (columns of W_UV)
  int32_t tail;  // tail variants only: positions L_b - tail .. L_b - 1 of every sequence
  int32_t weights;  // bf16 tail launcher: 0 = repack the weights into ws, then expand; 1 = repack only; 2 = ws already holds them
  float k_inv_scale, v_inv_scale;  // 8-bit tail variant only: 1 / scale of the two code planes
};

struct CompressArgs {
  CacheView expanded;  // all g groups
  CacheView latent;
  const int32_t* seq_lens;
  const void* w_inv;   // [r_kv][g*d_h], the cache's element type
  int32_t B, g, d_h, d_v, r_kv, d_r;
};

struct QuantizeArgs {
  CacheView src;  // 16-bit expanded cache
  CacheView dst;  // 8-bit expanded cache, same geometry and page ids
  const int32_t* seq_lens;
  int32_t B;
  float k_inv_scale, v_inv_scale;
};

struct AppendArgs {
  const void* rows;  // [B][s_q][row_bytes]
  CacheView latent;
  const int32_t* seq_lens;
  int32_t B, s_q, row_bytes;
};

struct RopeArgs {
  void* q_r;   // [B][s_q][h_q][d_r] or null
  void* rows;  // [B][s_q][row_elems], k_R at column r_kv; or null
  const int32_t* seq_lens;
  double log2_base;
  int32_t B, s_q, h_q, d_r, r_kv, row_elems;
};

struct OutProjArgs {
  const void* o;    // [M][K]
  const void* w_o;  // [D][K]
  void* y;          // [M][D]
  float* partial;   // [ksplit][M][D] when ksplit > 1
  int32_t M, K, D, ksplit, krange;
};

struct AbsorbQueryArgs {
  const void* q_c;
  const void* w_uk;
  void* q_hat;
  int32_t rows;  // B * s_q
  int32_t h_q, g, G, d_h, r_kv;
};

// Workspace layout (byte offsets) derived from a plan.
struct WsLayout {
  size_t table_off, first_slot_off, part_o_off, part_lse_off, total;
};

// Kernel launchers (each returns the hipError_t of its launch).
hipError_t launch_absorb_query_f32(const AbsorbQueryArgs&, hipStream_t);
hipError_t launch_absorb_query_bf16(const AbsorbQueryArgs&, hipStream_t);
hipError_t launch_decode_gqa_f32(const DecodeArgs&, hipStream_t);
hipError_t launch_decode_gqa_bf16(const DecodeArgs&, hipStream_t);
hipError_t launch_decode_absorb_f32(const DecodeArgs&, hipStream_t);
hipError_t launch_decode_absorb_bf16(const DecodeArgs&, hipStream_t);
hipError_t launch_combine_f32(const CombineArgs&, hipStream_t);                          // fp32 partials in d_h space, [chunks][M][d_v]
hipError_t launch_combine_gqa_bf16(const CombineArgs&, hipStream_t);                     // fp32 partials in d_h space, vector order (part_vec_index), bf16 out
hipError_t launch_combine_project_f32(const CombineArgs&, hipStream_t);                  // fp32 latent partials, fp32 out
hipError_t launch_combine_project_bf16(const CombineArgs&, hipStream_t);                 // bf16 latent partials, bf16 out
hipError_t launch_expand_f32(const ExpandArgs&, hipStream_t);
hipError_t launch_expand_bf16(const ExpandArgs&, void* ws /* packed weights, 2*group_count*r_kv*d_h bf16 */, hipStream_t);
hipError_t launch_expand_tail_f32(const ExpandArgs&, hipStream_t);
hipError_t launch_expand_tail_bf16(const ExpandArgs&, void* ws /* as above */, hipStream_t);
hipError_t launch_expand_fp8(const ExpandArgs&, void* ws /* as above */, hipStream_t);       // one-shot, `expanded` is an 8-bit cache
hipError_t launch_expand_tail_fp8(const ExpandArgs&, void* ws /* as above */, hipStream_t);  // `expanded` is an 8-bit cache
hipError_t launch_append_latent(const AppendArgs&, hipStream_t);
hipError_t launch_quantize_expanded(const QuantizeArgs&, hipStream_t);
hipError_t launch_quantize_latent(const QuantizeArgs&, hipStream_t);  // src: 16-bit latent cache, dst: 8-bit latent cache; k_inv_scale
hipError_t launch_decode_absorb_fp8(const DecodeArgs&, float c_scale, hipStream_t);  // the cache is an 8-bit latent cache
hipError_t launch_compress_f32(const CompressArgs&, hipStream_t);
hipError_t launch_compress_bf16(const CompressArgs&, hipStream_t);
hipError_t launch_rope_step(const RopeArgs&, bool bf16, hipStream_t);
hipError_t launch_out_proj_f32(const OutProjArgs&, hipStream_t);
hipError_t launch_out_proj_bf16(const OutProjArgs&, hipStream_t);
int out_proj_split(int M, int K, int D, int* krange);  // k-ranges of the bf16 kernel (needs D % 128 == 0, K % 256 == 0)
hipError_t launch_decode_gqa_fp8(const DecodeArgs&, float k_scale, float v_scale, hipStream_t);

hipError_t launch_probe_stream_read(const void* src, size_t bytes, uint32_t* sink, int blocks, hipStream_t);
hipError_t launch_probe_mfma(uint32_t* sink, int iters, int blocks, hipStream_t);

}  // namespace gqla

// The opaque plan of the public header.
struct gqla_plan {
  gqla_shape shape;
  int32_t path, page_size, num_cus, chunk_pages;
  std::vector<int32_t> lens;
  std::vector<gqla::ChunkEntry> chunks;
  std::vector<int32_t> first_slot;  // B + 1 entries
  gqla::WsLayout ws;
  const void* uploaded_ws;          // workspace the table was last uploaded into (host-side bookkeeping)
};
