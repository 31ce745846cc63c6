/*
 * gqla.h -- C ABI of the GQLA decode-attention library for AMD MI355X (gfx950).
 *
 * GQLA (Group-Query Latent Attention, paper Sec. 3.1) keeps one latent c_kv (r_kv elements) and one
 * shared RoPE key k_R (d_r elements) per cached token and indexes the up-projections W_UK, W_UV by
 * g KV groups.  The same weights give two algebraically equivalent decode paths:
 *
 *   MQA-absorb path (Sec. 3.1, "MQA-absorb path" equation):
 *       q_hat[i] = W_UK[j(i)] q_C[i];   logits = (q_hat[i].c_s + q_R[i].k_R,s) / sqrt(d_h + d_r);
 *       o_hat[i] = sum_s softmax_s(logits) c_s;   o[i] = W_UV[j(i)]^T o_hat[i]
 *   GQA path (Sec. 3.1, "GQA path" equation), over the expanded cache K_C = W_UK^T c, V = W_UV^T c:
 *       logits = (q_C[i].K_C[s, j(i)] + q_R[i].k_R,s) / sqrt(d_h + d_r);   o[i] = sum_s softmax_s(logits) V[s, j(i)]
 *
 * with head i routed to group j(i) = i / (h_q / g) (0-based form of the paper's ceil(i/(h_q/g));
 * heads j*G .. j*G+G-1 share group j, G = h_q / g).
 *
 * Conventions
 *   - All data pointers are DEVICE pointers unless a parameter says "host".  Structs passed by
 *     pointer (gqla_shape, gqla_cache) live in HOST memory and are read before the call returns.
 *   - Nothing here allocates, frees or synchronises device memory: the caller owns every buffer,
 *     including the workspace, and passes the hipStream_t (as void*) the kernels are enqueued on.
 *   - Every entry point validates its arguments on the host before launching anything and returns
 *     a gqla_status; no exceptions, no abort, nothing printed.  On any status other than GQLA_OK no
 *     kernel was launched by that call.  On GQLA_OK outputs are fully overwritten (asynchronously,
 *     in stream order).
 *   - s_q step tokens per sequence (1 = plain decode, 2 = one multi-token-prediction head).  The
 *     cached length L_b INCLUDES the s_q step tokens as its last rows; query t (0-based) sits at
 *     position L_b - s_q + t and attends to cached rows s <= L_b - s_q + t (causal inside the step).
 *   - dtype GQLA_BF16: caches, queries, weights, q_hat and out are bf16; all accumulation, softmax
 *     and the log-sum-exps are fp32 (split partials: fp32 on the GQA path, bf16 in latent space on the absorb
 *     path); QK^T and PV run on bf16 MFMA.  Shape limits of the MFMA
 *     kernels: (d_h, d_v) = (128, 128) or (192, 256) wherever an expanded cache is involved (see gqla_shape.d_v for
 *     the absorb path), d_r = 64, r_kv = 512, page_size a multiple of 64 (<= 1024).
 *     dtype GQLA_F32: everything fp32 on the vector ALU; d_h, d_v, d_r, r_kv, page_size multiples of 8, and
 *     d_h, d_v, r_kv at most 512 (GQLA_ERR_SHAPE beyond).
 *
 * Tensor layouts (row-major, last index fastest)
 *   q_c   [B][s_q][h_q][d_h]      q_r  [B][s_q][h_q][d_r]     q_hat [B][s_q][h_q][r_kv]
 *   w_uk  [g][r_kv][d_h]   w_uv  [g][r_kv][d_v]   (the transpose of the paper's d_h x r_kv head slice)
 *   out   [B][s_q][h_q][d_v]      lse  [B][s_q][h_q]  (fp32, natural log of the softmax denominator)
 *   (d_v = d_h unless the shape names a value dim of its own, d_h^V of Sec. 3.2.2)
 *
 * Cache pools (gqla_cache.pool): pages of page_size (P) tokens, back to back.
 *   latent page    [P][r_kv + d_r]           per token: c_kv | k_R           (Sec. 4.2.1: r_kv + d_r elements)
 *   expanded page, g_c groups (Sec. 4.2.2: 2 g d_h + d_r elements per token; g (d_h + d_v) + d_r with a value dim
 *   of its own), three planes of 8-element vectors so that every 16-byte vector is already an MFMA operand fragment:
 *       K_C : [g_c][d_h/8][P][8]     element (j, slot s, dim d) at ((j*(d_h/8) + d/8)*P + s)*8 + d%8
 *       V   : [g_c][P/8][d_v][8]     element (j, s, d) at g_c*P*d_h + ((j*(P/8) + s/8)*d_v + d)*8 + s%8
 *       k_R : [d_r/8][P][8]          element (s, d)    at g_c*P*(d_h + d_v) + ((d/8)*P + s)*8 + d%8
 *   Logical token t of sequence b lives in page  page_table[b*max_pages + t/P]  (or b*max_pages + t/P
 *   when page_table is NULL) at slot t % P.  Slots at or beyond L_b are never used by a decode call
 *   (whatever bits they hold) and never written by gqla_expand_cache.
 */
#ifndef GQLA_H
#define GQLA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GQLA_OK = 0,
  GQLA_ERR_NULL = 1,       /* a required pointer is NULL                                  */
  GQLA_ERR_SHAPE = 2,      /* dimensions unsupported or inconsistent (g does not divide h_q, ...) */
  GQLA_ERR_DTYPE = 3,      /* dtype not GQLA_F32 / GQLA_BF16, or not taken by this entry point */
  GQLA_ERR_ALIGN = 4,      /* a data pointer is not 16-byte aligned                         */
  GQLA_ERR_SEQLEN = 5,     /* some L_b < s_q, or L_b exceeds max_pages * page_size          */
  GQLA_ERR_PAGE = 6,       /* page_size / max_pages / num_pages inconsistent                */
  GQLA_ERR_WORKSPACE = 7,  /* workspace too small, or it does not hold this plan's table    */
  GQLA_ERR_DEVICE = 8,     /* a HIP call (copy or launch) failed                            */
  GQLA_ERR_PLAN = 9        /* plan was built for another shape / path                       */
} gqla_status;

typedef enum { GQLA_F32 = 0, GQLA_BF16 = 1 } gqla_dtype;
typedef enum { GQLA_PATH_ABSORB = 0, GQLA_PATH_GQA = 1 } gqla_path;

typedef struct {
  int32_t batch;   /* B   sequences in the step                              */
  int32_t h_q;     /*     query heads                                        */
  int32_t g;       /*     KV groups (divides h_q)                            */
  int32_t d_h;     /*     per-head content (key) dim                         */
  int32_t r_kv;    /*     latent rank                                        */
  int32_t d_r;     /*     decoupled-RoPE dim                                 */
  int32_t s_q;     /*     step tokens per sequence, 1 or 2                   */
  int32_t dtype;   /*     gqla_dtype                                         */
  float scale;     /*     softmax scale; 0 selects 1/sqrt(d_h + d_r) (Sec. 3.1) */
  int32_t d_v;     /*     per-head value dim d_h^V; 0 selects d_h.  A value dim of its own (the MLA checkpoints of
                          Sec. 3.2.2: d_h = 192, d_h^V = 256): w_uv is [g][r_kv][d_v], out [B][s_q][h_q][d_v], w_o
                          [d_model][h_q * d_v], the expanded cache's V plane has d_v dims.  GQLA_BF16: the absorb path
                          (gqla_absorb_query, gqla_decode_absorb and its 8-bit variant) takes d_h in {128, 192} and d_v
                          in {128, 256}; everything over a 16-bit expanded cache (gqla_expand_cache and its tail
                          variants, gqla_decode_gqa, gqla_compress_cache, plans for GQLA_PATH_GQA) takes (d_h, d_v) =
                          (128, 128) or (192, 256); the 8-bit expanded cache and gqla_select_path take (128, 128) only.
                          Other combinations: GQLA_ERR_SHAPE.  r_kv = 512, d_r = 64. */
} gqla_shape;

typedef struct {
  void* pool;                 /* device: num_pages pages in the format of the cache kind        */
  const int32_t* seq_lens;    /* device int32[batch]: L_b; read by the cache-update calls only  */
  const int32_t* page_table;  /* device int32[batch*max_pages], or NULL for the identity map    */
  int32_t page_size;          /* P, tokens per page                                            */
  int32_t max_pages;          /* row stride of page_table; every L_b <= max_pages * page_size  */
  int32_t num_pages;          /* pages in the pool; kernels skip (never dereference) ids outside [0, num_pages) */
  int32_t groups;             /* expanded cache: g_c groups stored per page; latent cache: ignored */
} gqla_cache;

/* ---- split plan (integer bookkeeping; the paper does not model paging or splitting, Sec. 5.1 (i)) ----
 *
 * A decode call cuts every sequence into chunks of whole pages, runs flash-decoding per chunk and merges
 * the chunk partials with a log-sum-exp combine.  The plan is a HOST object holding the chunk table.
 * Rule (all integer, reproduced bit for bit by the tests' independent implementation):
 *   npages_b = ceil(L_b / P);   slots = number of chunks the device works on at once:
 *       absorb: max(1, num_cus / ceil(h_q*s_q / 128))          gqa: max(1, num_cus*8 / (g * ceil(G*s_q / 32)))
 *       (gqa with a token team -- g = 1 and h_q*s_q <= 32, where the eight waves of a workgroup share one chunk:
 *       max(1, num_cus))
 *   chunk_pages = the cp in 1..max_b npages_b minimising, with n(cp) = sum_b ceil(npages_b/cp) chunks,
 *           w(cp) * ceil(n(cp) / slots) * (cp + ovh)  +  merge * ceil(max_b npages_b / cp),
 *       in eightieths of the time one page takes: ovh = 4 (absorb) or 2 (gqa; 16 with a token team) pages of
 *       per-chunk fixed cost;
 *       merge = 16 (absorb) or 5 (gqa) per chunk partial that the combine merges for the longest sequence;
 *       w(cp) = 80, except on the absorb path when the decode launch gives every 32 query rows a workgroup of their
 *       own and a page costs less: w(cp) = 53 if h_q*s_q <= 32 or 8*ceil(n(cp)/8) * ceil(h_q*s_q/32) <= num_cus;
 *       w(cp) = 10 on the gqa path with a token team;
 *       ties go to the larger cp;
 *   sequence b gets n_b = ceil(npages_b / chunk_pages) chunks of ceil(npages_b / n_b) pages (last one shorter);
 *   chunk k of b covers tokens [k*per_b*P, min((k+1)*per_b*P, L_b)) and owns partial slot first_slot[b] + k.
 */
typedef struct gqla_plan gqla_plan;

/* seq_lens_host: host int32[batch].  num_cus: compute units to plan for (256 on MI355X).  chunk_pages_override:
 * 0 = use the rule above, > 0 = force that chunk size (testing / tuning).  *out receives the plan. */
gqla_status gqla_plan_create(const gqla_shape* shape, const int32_t* seq_lens_host, int32_t page_size,
                             int32_t num_cus, int32_t path, int32_t chunk_pages_override, gqla_plan** out);
void gqla_plan_destroy(gqla_plan* plan);
int32_t gqla_plan_num_chunks(const gqla_plan* plan);
int32_t gqla_plan_chunk_pages(const gqla_plan* plan);
/* Copies up to *n chunk triples (b, tok_begin, tok_end) in slot order to triples (host int32[3 * *n]) and the
 * per-sequence first slots to first_slot (host int32[batch], may be NULL); sets *n to the chunk count. */
gqla_status gqla_plan_export(const gqla_plan* plan, int32_t* triples, int32_t* first_slot, int32_t* n);
/* Bytes of device workspace a decode call with this plan needs: the chunk table, then the partial outputs (GQA path:
 * d_v fp32 values per chunk and row; absorb path: r_kv values, bf16 for GQLA_BF16 and fp32 for GQLA_F32; with
 * GQLA_BF16 the rows are rounded up to whole blocks of 32 and the order is the library's own) and the fp32 partial
 * log-sum-exps [chunks][s_q*h_q]. */
size_t gqla_plan_workspace_bytes(const gqla_plan* plan);
/* Enqueues the copy of the plan's chunk table into the head of ws (device, 16-byte aligned, at least
 * gqla_plan_workspace_bytes).  Must precede, in stream order, every decode call that uses (plan, ws).  The plan
 * must stay alive until that copy has executed. */
gqla_status gqla_plan_upload(gqla_plan* plan, void* ws, size_t ws_bytes, void* stream);

/* ---- the decode paths --------------------------------------------------------------------------------- */

/* Query absorption, first line of the MQA-absorb equation (Sec. 3.1): q_hat[b,t,i,:] = W_UK[j(i)] q_c[b,t,i,:]
 * (an r_kv-vector per head).  q_r is not touched (it passes through to gqla_decode_absorb). */
gqla_status gqla_absorb_query(const gqla_shape* shape, const void* q_c, const void* w_uk, void* q_hat,
                              void* stream);

/* MQA-absorb decode (Sec. 3.1, MQA-absorb equation, lines 2-6): split-L flash-decoding of all h_q*s_q rows
 * over the latent cache, each chunk's latent-space output projected through W_UV[j(i)], then the log-sum-exp
 * combine.  plan: built with GQLA_PATH_ABSORB for this shape and the lengths in the cache, uploaded into ws.
 * lse may be NULL. */
gqla_status gqla_decode_absorb(const gqla_shape* shape, const gqla_plan* plan, const void* q_hat,
                               const void* q_r, const gqla_cache* latent, const void* w_uv, void* out,
                               float* lse, void* ws, size_t ws_bytes, void* stream);

/* Cache switch latent -> expanded (Sec. 3.1, "Two equivalent decoding paths": the one-shot expand; K_C = W_UK^T c,
 * V = W_UV^T c per group, k_R copied).  Expands groups [group_begin, group_begin + group_count) of every token
 * t < L_b (L_b read from latent->seq_lens on the device) into `expanded`, whose pages hold
 * expanded->groups == group_count groups and which must use the same page_size, max_pages and page ids
 * (page_table content) as `latent`.  A slice with group_count < g is one rank's share of head-axis
 * tensor parallelism.  `ws` is device scratch of at least gqla_expand_workspace_bytes(shape, group_count) bytes
 * (16-byte aligned; it receives the slice's weights reordered for the matrix cores and may be reused or freed
 * once the call's kernels have run); with dtype GQLA_F32 no scratch is needed and ws may be NULL.
 * Errors: GQLA_ERR_SHAPE for a group range outside [0, g) or expanded->groups != group_count, GQLA_ERR_PAGE when
 * the two caches disagree on geometry, GQLA_ERR_WORKSPACE when ws is NULL or too small. */
gqla_status gqla_expand_cache(const gqla_shape* shape, const gqla_cache* latent, const void* w_uk,
                              const void* w_uv, int32_t group_begin, int32_t group_count,
                              const gqla_cache* expanded, void* ws, size_t ws_bytes, void* stream);
/* Bytes of scratch gqla_expand_cache needs for a slice of group_count groups: group_count * r_kv * (d_h + d_v) * 2
 * (0 for GQLA_F32 or a bad shape). */
size_t gqla_expand_workspace_bytes(const gqla_shape* shape, int32_t group_count);

/* ---- the per-step cache updates around the two decode paths (Sec. 3.1: each step caches the new token's c_kv and
 * shared RoPE key; the GQA path's K_C, V of that token follow from the same latent) ----
 *
 * gqla_append_latent writes the step's rows into the latent cache: rows is device memory [B][s_q][r_kv + d_r]
 * (c_kv | k_R per token, the cache's element type); row t of sequence b goes to logical position L_b - s_q + t, with
 * L_b read from latent->seq_lens on the device, i.e. the lengths already count the step's tokens, as the decode calls
 * expect them.  A sequence with L_b < s_q only receives the rows that have a position >= 0.  Nothing else is written.
 *
 * gqla_expand_cache_tail is gqla_expand_cache restricted to the last tail_tokens positions of every sequence
 * (L_b - tail_tokens .. L_b - 1, clipped at 0): after gqla_append_latent with s_q = tail_tokens it brings an
 * expanded cache that was complete before the step up to date, at a cost that does not grow with the context.
 * Arguments, geometry rules, scratch and errors as for gqla_expand_cache; tail_tokens must be in [1, page_size]
 * (GQLA_ERR_SHAPE otherwise).  Both calls only enqueue work on `stream`. */
gqla_status gqla_append_latent(const gqla_shape* shape, const void* rows, const gqla_cache* latent, void* stream);
gqla_status gqla_expand_cache_tail(const gqla_shape* shape, const gqla_cache* latent, const void* w_uk,
                                   const void* w_uv, int32_t group_begin, int32_t group_count,
                                   const gqla_cache* expanded, int32_t tail_tokens, void* ws, size_t ws_bytes,
                                   void* stream);

/* The step's expansion with the weights repacked ahead of time.  gqla_expand_cache and gqla_expand_cache_tail first
 * reorder the slice's W_UK, W_UV into the operand order of the matrix instructions, in the caller's scratch; a serving
 * loop, whose weights do not change, does that once: gqla_pack_expand_weights writes the reordered copy of groups
 * group_begin .. group_begin + group_count - 1 into `packed` (device memory, 16-byte aligned, at least
 * gqla_expand_workspace_bytes(shape, group_count) bytes; the layout is the library's own and holds for this build and
 * this shape only), and gqla_expand_cache_tail_packed is gqla_expand_cache_tail reading that copy -- same results bit
 * for bit, one kernel less per step.  GQLA_BF16 only (GQLA_ERR_DTYPE otherwise: the fp32 kernels read the weights as they
 * are); `packed` must stay untouched between the two calls; other arguments, geometry rules and errors as for
 * gqla_expand_cache_tail (GQLA_ERR_WORKSPACE when packed_bytes is too small).  Both calls only enqueue work on `stream`. */
gqla_status gqla_pack_expand_weights(const gqla_shape* shape, const void* w_uk, const void* w_uv, int32_t group_begin,
                                     int32_t group_count, void* packed, size_t packed_bytes, void* stream);
gqla_status gqla_expand_cache_tail_packed(const gqla_shape* shape, const gqla_cache* latent, const void* packed,
                                          size_t packed_bytes, int32_t group_count, const gqla_cache* expanded,
                                          int32_t tail_tokens, void* stream);

/* gqla_expand_cache_tail for callers that cannot allocate device memory at all (code recorded into a HIP graph, tight
 * serving loops, harnesses that forbid hipMalloc): same operation, same results bit for bit, but the scratch (the
 * slice's weights in matrix-core order) lives in a fixed 2 MiB device array inside the library instead of a
 * caller-supplied workspace, and the call allocates and frees nothing.  Every GPU the process uses holds its own copy of
 * that array until the process ends.  Limit: gqla_expand_workspace_bytes(shape, group_count) must not exceed
 * gqla_expand_cache_tail_static_max_workspace() (2 MiB: up to 8 groups at r_kv = 512, d_h = d_v = 128 in bf16, up to 4 at d_h = 192, d_v = 256);
 * GQLA_ERR_WORKSPACE beyond that, before anything is launched.  All calls on one GPU share the array: two such calls
 * whose kernels can overlap (different streams without an ordering between them) race on it; calls on one stream, or
 * ordered by events, are safe.  The array keeps the previous call's content; each call overwrites the part it uses
 * before reading it.  Other arguments and errors as for gqla_expand_cache_tail; GQLA_ERR_DEVICE if the array's address
 * cannot be obtained on the current device. */
gqla_status gqla_expand_cache_tail_static(const gqla_shape* shape, const gqla_cache* latent, const void* w_uk,
                                          const void* w_uv, int32_t group_begin, int32_t group_count,
                                          const gqla_cache* expanded, int32_t tail_tokens, void* stream);
size_t gqla_expand_cache_tail_static_max_workspace(void);

/* GQA-path decode (Sec. 3.1, GQA-path equation) over an expanded cache holding expanded->groups == shape->g
 * groups (for a tensor-parallel slice pass a shape with h_q and g already divided).  plan: built with
 * GQLA_PATH_GQA, uploaded into ws.  lse may be NULL. */
gqla_status gqla_decode_gqa(const gqla_shape* shape, const gqla_plan* plan, const void* q_c, const void* q_r,
                            const gqla_cache* expanded, void* out, float* lse, void* ws, size_t ws_bytes,
                            void* stream);

/* ---- the steps either side of the path: rotary embedding of the step's inputs, output projection ------------------
 * gqla_rope_step applies rope_t (Sec. 3.1, "Architecture": q^R_{t,i} = rope_t(.), k^R_t = rope_t(.)) IN PLACE to the
 * step's un-rotated vectors: q_r [B][s_q][h_q][d_r] (every head) and the k_R part (columns r_kv .. r_kv + d_r - 1) of
 * rows [B][s_q][r_kv + d_r], the rows gqla_append_latent takes; either pointer may be NULL (not both).  Step token i of
 * sequence b has position t = L_b - s_q + i, L_b read from seq_lens (device memory, int32[B], the lengths that already
 * count the step's tokens); tokens with t < 0 are left alone.  The paper takes the rotary embedding over from MLA
 * without restating it; this library uses the published form: d_r/2 adjacent pairs (x[2p], x[2p+1]), pair p turned by
 * the angle t * rope_base^(-2p/d_r) (the angle is formed and reduced modulo a full turn in double precision; sine,
 * cosine and the rotation are fp32, the result rounded to the element type).  Errors: GQLA_ERR_SHAPE unless rope_base is finite and > 1, d_r and r_kv are even and d_r <= 512.
 *
 * gqla_output_projection computes y_t = W^O [o_{t,1}; ...; o_{t,h_q}] (last line of the GQA-path and of the MQA-absorb
 * equation): o is a decode call's output [B][s_q][h_q][d_h], w_o is [d_model][h_q * d_h] row-major (the paper's
 * W^O in R^{D x h_q d_h}), y is [B][s_q][d_model]; all device memory of the shape's element type, fp32 accumulation.
 * With GQLA_BF16, d_model must be a multiple of 128 and h_q * d_h of 256, at most 2^24 (GQLA_ERR_SHAPE otherwise), and the call may
 * need device scratch: ws of at least gqla_output_projection_workspace_bytes(shape, d_model) bytes, 16-byte aligned
 * (fp32 partial sums over ranges of the contraction, added in a fixed order; GQLA_ERR_NULL / GQLA_ERR_WORKSPACE when
 * it is needed and missing or too small).  GQLA_F32 needs none.  Both calls only enqueue work on `stream`. */
gqla_status gqla_rope_step(const gqla_shape* shape, const int32_t* seq_lens, float rope_base, void* q_r, void* rows,
                           void* stream);
gqla_status gqla_output_projection(const gqla_shape* shape, int32_t d_model, const void* o, const void* w_o, void* y,
                                   void* ws, size_t ws_bytes, void* stream);
size_t gqla_output_projection_workspace_bytes(const gqla_shape* shape, int32_t d_model);

/* ---- cache compression: the reverse switch (Sec. 3.1: the cache is converted once, in either direction, at deployment) ----
 * The expansion k^C = A c, A = [W_UK[0]^T; ...; W_UK[g-1]^T] in R^{g d_h x r_kv}, can be undone when A has full column
 * rank (needs g d_h >= r_kv): c = A^+ k^C with the left inverse A^+ = (A^T A)^{-1} A^T in R^{r_kv x g d_h}.
 * gqla_left_inverse computes A^+ on the HOST (both arguments host memory, fp32: w_uk_host [g][r_kv][d_h], w_inv_host
 * [r_kv][g*d_h], columns ordered group-major, dim-minor like k^C), in double precision through the Cholesky factor of
 * A^T A; GQLA_ERR_SHAPE when g d_h < r_kv or A^T A is not positive definite (a Cholesky pivot at or below 1e-12 of
 * its diagonal entry).  gqla_compress_cache applies a left inverse
 * (device memory, the cache's element type, same layout) to the K_C plane of every token t < L_b of `expanded` (all g
 * groups; L_b read from expanded->seq_lens on the device) and writes c_kv | k_R into `latent`, which must use the same
 * page_size, max_pages and page ids.  On a cache whose keys were rounded to 16 bits the result is the least-squares
 * latent of the rounded keys. */
gqla_status gqla_left_inverse(const gqla_shape* shape, const float* w_uk_host, float* w_inv_host);
gqla_status gqla_compress_cache(const gqla_shape* shape, const gqla_cache* expanded, const void* w_inv,
                                const gqla_cache* latent, void* stream);

/* ---- 8-bit expanded cache for the GQA path --------------------------------------------------------------
 * The paper names quantised KV caches as complementary to the method and leaves them out of its model (Sec. 2
 * "Related work"; Sec. 5.1, item (i)); format and scales are this library's.  K_C and V are stored as E4M3 codes of
 * the OCP 8-bit floating point specification ("FN" variant: bias 7, 3 mantissa bits, subnormals, no infinities,
 * largest finite value 448), one positive scale per tensor kind:
 *     code = E4M3(fp32(x) * fp32(1 / scale))   round to nearest, ties to even, magnitudes above 448 saturate
 *     x'   = value(code) * scale
 * k_R stays in 16 bits; queries, outputs and the latent cache are GQLA_BF16 (GQLA_ERR_DTYPE otherwise).  A page of P
 * tokens and g_c groups has P * (2 g_c d_h + 2 d_r) BYTES; every 16-byte vector of the two code planes holds what
 * one lane of a 32x32x16 matrix instruction consumes in two consecutive k-steps (byte offsets inside the page):
 *     K8 : [g_c][d_h/16][P][16]      dim d = 32 kp + 16 u + 8 h + i  ->  ((j*(d_h/16) + 2 kp + h)*P + s)*16 + 8 u + i
 *     V8 : [g_c][P/32][d_h][2][16]   slot s = 32 T + 16 u + 8 h + i  ->  g_c*P*d_h + (((j*(P/32) + T)*d_h + d)*2 + h)*16 + 8 u + i
 *     k_R: [d_r/8][P][8] 16-bit      2*g_c*P*d_h + (((d/8)*P + s)*8 + d%8)*2
 * gqla_quantize_expanded converts an expanded cache of the 16-bit format (all groups it holds, every token t < L_b,
 * L_b read from expanded->seq_lens on the device) into an 8-bit one with the same page geometry and page ids; bytes of
 * slots no token owns are left as they are.  gqla_decode_gqa_fp8 is gqla_decode_gqa over such a cache (same plan,
 * workspace and outputs): the codes are widened to bf16 in registers, the scales applied to the content part of the
 * logits and to the output.  Errors as for the 16-bit calls; scales that are not positive and finite: GQLA_ERR_SHAPE. */
gqla_status gqla_quantize_expanded(const gqla_shape* shape, const gqla_cache* expanded, const gqla_cache* expanded_fp8,
                                   float k_scale, float v_scale, void* stream);
gqla_status gqla_decode_gqa_fp8(const gqla_shape* shape, const gqla_plan* plan, const void* q_c, const void* q_r,
                                const gqla_cache* expanded_fp8, float k_scale, float v_scale, void* out, float* lse,
                                void* ws, size_t ws_bytes, void* stream);
/* gqla_expand_cache_tail whose destination is an 8-bit cache: the step's positions of every sequence, with the codes
 * that expanding into a 16-bit cache and converting it would give (each result is rounded to bf16 before it is
 * quantised).  Arguments and errors as for gqla_expand_cache_tail, plus the two scales. */
gqla_status gqla_expand_cache_tail_fp8(const gqla_shape* shape, const gqla_cache* latent, const void* w_uk,
                                       const void* w_uv, int32_t group_begin, int32_t group_count,
                                       const gqla_cache* expanded_fp8, int32_t tail_tokens, float k_scale, float v_scale,
                                       void* ws, size_t ws_bytes, void* stream);
/* gqla_expand_cache whose destination is an 8-bit cache (every token t < L_b): the cache switch latent -> 8-bit expanded
 * in one pass, with the codes that gqla_expand_cache followed by gqla_quantize_expanded would give, at half the bytes
 * written and without the 16-bit intermediate.  Arguments and errors as for gqla_expand_cache, plus the two scales. */
gqla_status gqla_expand_cache_fp8(const gqla_shape* shape, const gqla_cache* latent, const void* w_uk, const void* w_uv,
                                  int32_t group_begin, int32_t group_count, const gqla_cache* expanded_fp8, float k_scale,
                                  float v_scale, void* ws, size_t ws_bytes, void* stream);
int64_t gqla_expanded_fp8_bytes_per_token(int32_t groups, int32_t d_h, int32_t d_r);

/* ---- 8-bit latent cache for the MQA-absorb path ----------------------------------------------------------
 * The same reading (Sec. 2; Sec. 5.1, item (i): quantised caches are complementary, no format given) applied to the
 * cache of Sec. 4.2.1: c_kv as E4M3 codes with ONE positive scale for the whole cache (conversion rule as above),
 * k_R kept in 16 bits.  A token takes r_kv + 2 d_r bytes (640 at r_kv 512, d_r 64, against 1152).  A page of P tokens
 * (byte offsets inside the page of P * (r_kv + 2 d_r) bytes):
 *     codes : [P][r_kv]          s * r_kv + d
 *     k_R   : [P][d_r] 16-bit    P * r_kv + (s * d_r + d) * 2
 * gqla_quantize_latent converts a 16-bit latent cache (every token t < L_b, L_b read from latent->seq_lens on the
 * device) into an 8-bit one with the same page geometry and page ids (each cache may have its own page table); bytes
 * of slots no token owns are left as they are.  gqla_decode_absorb_fp8 is gqla_decode_absorb over such a cache (same
 * plan, workspace and outputs): the MQA-absorb equation (Sec. 3.1) with keys [c'; k_R] and values c', c' = value(code)
 * * c_scale; the codes are widened to bf16 (exactly) on their way into LDS, the scale is applied to the content part
 * of the logits and to the output.  GQLA_BF16 shapes only (GQLA_ERR_DTYPE otherwise); a scale that is not positive and
 * finite: GQLA_ERR_SHAPE; other errors as for gqla_decode_absorb. */
gqla_status gqla_quantize_latent(const gqla_shape* shape, const gqla_cache* latent, const gqla_cache* latent_fp8,
                                 float c_scale, void* stream);
gqla_status gqla_decode_absorb_fp8(const gqla_shape* shape, const gqla_plan* plan, const void* q_hat, const void* q_r,
                                   const gqla_cache* latent_fp8, float c_scale, const void* w_uv, void* out, float* lse,
                                   void* ws, size_t ws_bytes, void* stream);
int64_t gqla_latent_fp8_bytes_per_token(int32_t r_kv, int32_t d_r);

/* ---- sizes and diagnostics ------------------------------------------------------------------------------ */
/* Elements per token of the two caches (Sec. 4.2.1: r_kv + d_r;  Sec. 4.2.2: 2 g d_h + d_r). */
int64_t gqla_latent_elems_per_token(int32_t r_kv, int32_t d_r);
int64_t gqla_expanded_elems_per_token(int32_t groups, int32_t d_h, int32_t d_r);
/* Element offsets inside a pool (the formulas in the header comment), for callers that fill caches themselves. */
int64_t gqla_latent_offset(int64_t page, int32_t slot, int32_t col, int32_t page_size, int32_t r_kv, int32_t d_r);
int64_t gqla_expanded_k_offset(int64_t page, int32_t j, int32_t slot, int32_t d, int32_t page_size, int32_t groups, int32_t d_h, int32_t d_r);
int64_t gqla_expanded_v_offset(int64_t page, int32_t j, int32_t slot, int32_t d, int32_t page_size, int32_t groups, int32_t d_h, int32_t d_r);
int64_t gqla_expanded_kr_offset(int64_t page, int32_t slot, int32_t d, int32_t page_size, int32_t groups, int32_t d_h, int32_t d_r);
/* The same for an expanded cache whose value dim differs from its key dim (d_h^V of Sec. 3.2.2; d in [0, d_v) for the V
 * plane); with d_v = d_h they return what the functions above return. */
int64_t gqla_expanded_elems_per_token_dv(int32_t groups, int32_t d_h, int32_t d_v, int32_t d_r);
int64_t gqla_expanded_k_offset_dv(int64_t page, int32_t j, int32_t slot, int32_t d, int32_t page_size, int32_t groups, int32_t d_h, int32_t d_v, int32_t d_r);
int64_t gqla_expanded_v_offset_dv(int64_t page, int32_t j, int32_t slot, int32_t d, int32_t page_size, int32_t groups, int32_t d_h, int32_t d_v, int32_t d_r);
int64_t gqla_expanded_kr_offset_dv(int64_t page, int32_t slot, int32_t d, int32_t page_size, int32_t groups, int32_t d_h, int32_t d_v, int32_t d_r);

/* Path selection: one set of weights serves both paths and the serving runtime picks, per device, the one its
 * hardware runs faster (Abstract); the two-roof time model that decides it is Sec. 4.2.3.  The paper's Roofline
 * model of one decode step over `cached_tokens` tokens (summed over the batch): the absorb path moves
 * 2(r_kv + d_r) bytes and performs 2 h_q s_q (2 r_kv + d_r) FLOPs per cached token (Sec. 4.2.1), the GQA path
 * 2(2 g d_h + d_r) bytes and 2 h_q s_q (2 d_h + d_r) FLOPs (Sec. 4.2.2); the predicted time of a path is
 * max(bytes / hbm_bytes_per_s, flops / mfma_flops_per_s) (Sec. 4.2.3).  Element size: 2 bytes for GQLA_BF16, 4 for
 * GQLA_F32.  Pure host arithmetic; the two rates are whatever the caller trusts (published peaks, or the rates the
 * probes below measure).  faster_path is the gqla_path with the smaller predicted time (absorb on a tie). */
typedef struct {
  double absorb_bytes, absorb_flops, absorb_intensity, absorb_seconds;
  double gqa_bytes, gqa_flops, gqa_intensity, gqa_seconds;
  double ridge;          /* mfma_flops_per_s / hbm_bytes_per_s (Sec. 4.1) */
  int32_t faster_path;   /* gqla_path */
} gqla_path_estimate;
gqla_status gqla_estimate_paths(const gqla_shape* shape, int64_t cached_tokens, double hbm_bytes_per_s,
                                double mfma_flops_per_s, gqla_path_estimate* out);

/* The same choice for THIS library's kernels on the MI355X (GQLA_BF16 only; GQLA_ERR_DTYPE otherwise): the paper's
 * two-roof form with the rates the kernels sustain instead of the chip's peaks and a fixed cost per call, and, for
 * the absorb path, the critical path of one workgroup when the batch is too small to fill the chip.  All constants are
 * measurements of this build (the operating-point, batch-sweep and all-config tables under profiles/):
 *   absorb (query absorption + decode):  24 us + max(bytes / 5.5 TB/s, flops / 1.09 PFLOP/s, rounds * (per + 4) * page)
 *          where the split-plan rule of gqla_plan_create, applied to `batch` sequences of cached_tokens / batch tokens
 *          on 64-token pages and 256 compute units, gives every workgroup `rounds` chunks of `per` pages, and a page
 *          costs a workgroup 3.8 us (1.6 us when h_q s_q <= 32; 2.6 us when 8 * ceil(chunks / 8) * ceil(h_q s_q / 32) <= 256,
 *          where the launch gives every 32 rows their own workgroup; else 3.0 us when h_q s_q <= 64)
 *   gqa    (decode on the expanded cache): 26 us + min(f bytes, 200 MB) / 10 TB/s + max(0, f bytes - 200 MB) / 7.0 TB/s,
 *          f = 1 + 0.05 * (ceil(G s_q / 32) - 1): a cache of up to 200 MB is still in the chip's last-level cache from
 *          the step before; a group with 64 query rows costs a few percent more per byte (a wave takes both row blocks)
 * with bytes and flops as in gqla_estimate_paths.  faster_path is the path with the smaller time (absorb on a tie). */
typedef struct {
  double absorb_seconds, gqa_seconds;
  int32_t faster_path;   /* gqla_path */
} gqla_path_choice;
gqla_status gqla_select_path(const gqla_shape* shape, int64_t cached_tokens, gqla_path_choice* out);

/* Ceiling probes (measurement only; they compute nothing of the method).  The caller times them with events on
 * `stream` and derives  bytes / t  resp.  gqla_probe_mfma_flops(iters, num_cus) / t.
 *   gqla_probe_stream_read: every byte of src[0, bytes) is read once with 16-byte loads by 8 * num_cus workgroups;
 *     bytes must be a multiple of 16 * 1024 * 8 * num_cus (GQLA_ERR_SHAPE otherwise).  `sink` is 4 bytes of device
 *     memory that is (practically) never written.
 *   gqla_probe_mfma_bf16: num_cus workgroups of 4 waves issue 4 * iters independent-accumulator
 *     v_mfma_f32_32x32x16_bf16 each, operands resident in registers with random sign and mantissa bits. */
gqla_status gqla_probe_stream_read(const void* src, size_t bytes, void* sink, int32_t num_cus, void* stream);
gqla_status gqla_probe_mfma_bf16(void* sink, int32_t iters, int32_t num_cus, void* stream);
double gqla_probe_mfma_flops(int32_t iters, int32_t num_cus);

/* Kernel timing (measurement only).  A decode call launches two kernels, the split-L decode kernel and the small
 * combine; events placed around the call time both.  After gqla_time_next_decode_kernel(event_begin, event_end) -- two
 * hipEvent_t created by the caller with timing enabled, passed as void* -- the NEXT gqla_decode_absorb, gqla_decode_gqa
 * or gqla_decode_gqa_fp8 call made by the same host thread records event_begin immediately before and event_end
 * immediately after its split-L decode kernel, on the call's stream; the pair is then forgotten (one call only; a call
 * that fails its argument checks still consumes it once it got past them).  Two NULLs forget a pending pair;
 * one NULL is GQLA_ERR_NULL.  The library keeps no reference to the events after that decode call returns. */
gqla_status gqla_time_next_decode_kernel(void* event_begin, void* event_end);

const char* gqla_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* GQLA_H */
