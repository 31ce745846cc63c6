// Host side of the GQLA library: argument validation, the integer split plan, workspace layout and the
// extern "C" entry points declared in gqla.h.  No device memory is allocated here.
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>

#include "gqla_internal.h"

using namespace gqla;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// per-head value dim (0 in the struct selects d_h)
int32_t value_dim(const gqla_shape* s) { return s->d_v > 0 ? s->d_v : s->d_h; }

gqla_status check_shape(const gqla_shape* s) {
  if (!s) return GQLA_ERR_NULL;
  if (s->dtype != GQLA_F32 && s->dtype != GQLA_BF16) return GQLA_ERR_DTYPE;
  if (s->batch < 0 || s->h_q <= 0 || s->g <= 0 || s->h_q % s->g != 0) return GQLA_ERR_SHAPE;
  if (s->s_q != 1 && s->s_q != 2) return GQLA_ERR_SHAPE;
  if (s->d_h <= 0 || s->r_kv <= 0 || s->d_r <= 0 || s->d_v < 0) return GQLA_ERR_SHAPE;
  const int32_t d_v = value_dim(s);
  if (!(s->scale >= 0.f) || std::isinf(s->scale)) return GQLA_ERR_SHAPE;
  if (s->dtype == GQLA_BF16) {
    if ((s->d_h != 128 && s->d_h != 192) || (d_v != 128 && d_v != 256) || s->d_r != 64 || s->r_kv != 512) return GQLA_ERR_SHAPE;
  } else {
    if (s->d_h % 8 || d_v % 8 || s->d_r % 8 || s->r_kv % 8 || s->d_h > 512 || d_v > 512 || s->r_kv > 512) return GQLA_ERR_SHAPE;
  }
  return GQLA_OK;
}

// The 16-bit expanded cache and what reads or writes it (GQA path, the cache switches in both directions): in bf16 the
// kernels exist for (d_h, d_v) = (128, 128) and (192, 256) (the shape of Sec. 3.2.2); fp32 takes any dims.
gqla_status check_shape_expanded(const gqla_shape* s) {
  const gqla_status st = check_shape(s);
  if (st != GQLA_OK) return st;
  if (s->dtype == GQLA_BF16) {
    const int32_t d_v = value_dim(s);
    if (!((s->d_h == 128 && d_v == 128) || (s->d_h == 192 && d_v == 256))) return GQLA_ERR_SHAPE;
  }
  return GQLA_OK;
}

// The 8-bit expanded cache (and the calibrated path choice) is built for equal key and value dims of 128.
gqla_status check_shape_equal_dims(const gqla_shape* s) {
  const gqla_status st = check_shape(s);
  if (st != GQLA_OK) return st;
  if (value_dim(s) != s->d_h || (s->dtype == GQLA_BF16 && s->d_h != 128)) return GQLA_ERR_SHAPE;
  return GQLA_OK;
}

gqla_status check_page_size(const gqla_shape* s, int32_t page_size) {
  if (page_size <= 0) return GQLA_ERR_PAGE;
  if (s->dtype == GQLA_BF16) {
    if (page_size % 64 || page_size > 1024) return GQLA_ERR_PAGE;
  } else if (page_size % 8) {
    return GQLA_ERR_PAGE;
  }
  return GQLA_OK;
}

float resolved_scale(const gqla_shape* s) {
  return s->scale > 0.f ? s->scale : 1.0f / std::sqrt((float)(s->d_h + s->d_r));
}

bool same_shape(const gqla_shape& a, const gqla_shape& b) {
  return a.batch == b.batch && a.h_q == b.h_q && a.g == b.g && a.d_h == b.d_h && a.r_kv == b.r_kv &&
         a.d_r == b.d_r && a.s_q == b.s_q && a.dtype == b.dtype && value_dim(&a) == value_dim(&b);
}

gqla_status check_cache(const gqla_shape* s, const gqla_cache* c, int32_t page_size, int32_t max_len) {
  if (!c || !c->pool) return GQLA_ERR_NULL;
  if (!aligned16(c->pool) || (c->page_table && (reinterpret_cast<uintptr_t>(c->page_table) & 3u))) return GQLA_ERR_ALIGN;
  if (c->page_size != page_size || c->max_pages <= 0 || c->num_pages <= 0) return GQLA_ERR_PAGE;
  if ((int64_t)c->max_pages * c->page_size < max_len) return GQLA_ERR_SEQLEN;
  if (!c->page_table && (int64_t)c->num_pages < (int64_t)s->batch * c->max_pages) return GQLA_ERR_PAGE;
  return GQLA_OK;
}

// GQA path, one group with at most 32 query rows (one rank's share of head-axis tensor parallelism): a chunk would
// be a single wave's work; instead the eight waves of a workgroup take every eighth tile of one chunk each and merge
// their partials before anything is written.
bool gqa_token_team(const gqla_shape& s) { return s.g == 1 && (int64_t)s.h_q * s.s_q <= 32; }

int32_t plan_slots(const gqla_shape& s, int32_t num_cus, int32_t path) {
  if (path == GQLA_PATH_ABSORB) {
    const int32_t rb = (int32_t)ceil_div((int64_t)s.h_q * s.s_q, 128);
    return std::max(1, num_cus / rb);
  }
  const int32_t rb = (int32_t)ceil_div((int64_t)(s.h_q / s.g) * s.s_q, 32);
  if (gqa_token_team(s)) return std::max(1, num_cus);  // the eight waves of a workgroup share one chunk
  return std::max<int64_t>(1, (int64_t)num_cus * 8 / ((int64_t)s.g * rb));
}

// Chunk size of the split plan (the rule documented in gqla.h).  Cost of a candidate cp, in eightieths of the time a
// 128-row absorb workgroup (or a GQA wave) spends on one page: rounds of chunks on the device, each a chunk plus its
// fixed cost, then the combine, whose time is set by the longest chain of chunk partials it merges for one sequence.
// On the absorb path a page costs 53 instead of 80 when the launch gives every 32 query rows a workgroup of their own
// (at most 32 rows per sequence, or so few chunks that all those workgroups run at once).  On the GQA path with a token
// team a page costs the workgroup an eighth (10), and the fixed cost counts eight times as many pages (16).
int32_t choose_chunk_pages(const std::vector<int32_t>& npages, const gqla_shape& s, int32_t num_cus, int32_t path) {
  int32_t max_np = 1;
  for (int32_t v : npages) max_np = std::max(max_np, v);
  const int64_t slots = plan_slots(s, num_cus, path);
  const bool team = path == GQLA_PATH_GQA && gqa_token_team(s);
  const int64_t ovh = path == GQLA_PATH_ABSORB ? 4 : (team ? 16 : 2);
  const int64_t merge = path == GQLA_PATH_ABSORB ? 16 : 5;
  const int64_t M = (int64_t)s.h_q * s.s_q;
  int64_t best = -1;
  int32_t cp = 1;
  for (int32_t c = 1; c <= max_np; ++c) {
    int64_t n = 0;
    for (int32_t v : npages) n += ceil_div(v, c);
    const bool shared_rows = path == GQLA_PATH_ABSORB && (M <= 32 || ceil_div(n, 8) * 8 * ceil_div(M, 32) <= num_cus);
    const int64_t weight = team ? 10 : (shared_rows ? 53 : 80);
    const int64_t cost = weight * ceil_div(n, slots) * (c + ovh) + merge * ceil_div(max_np, c);
    if (best < 0 || cost <= best) {
      best = cost;
      cp = c;
    }
  }
  return cp;
}

WsLayout make_layout(const gqla_plan& p) {
  WsLayout w;
  const size_t n = p.chunks.size();
  const size_t M = (size_t)p.shape.s_q * p.shape.h_q;
  w.table_off = 0;
  w.first_slot_off = align_up(n * sizeof(ChunkEntry), 16);
  w.part_o_off = align_up(w.first_slot_off + (p.shape.batch + 1) * sizeof(int32_t), 256);
  size_t po;
  if (p.path == GQLA_PATH_GQA) po = n * (p.shape.dtype == GQLA_BF16 ? (M + 31) / 32 * 32 : M) * value_dim(&p.shape) * 4;   // bf16 kernels: whole blocks of 32 rows
  else if (p.shape.dtype == GQLA_BF16) po = n * ((M + 31) / 32 * 32) * p.shape.r_kv * 2;   // whole blocks of 32 rows (part_vec_index)
  else po = n * M * p.shape.r_kv * 4;
  w.part_lse_off = align_up(w.part_o_off + po, 256);
  w.total = align_up(w.part_lse_off + n * M * 4, 256);
  return w;
}

gqla_status check_decode_common(const gqla_shape* shape, const gqla_plan* plan, int32_t path, const gqla_cache* cache,
                                const void* qa, const void* qr, const void* out, const float* lse, const void* ws,
                                size_t ws_bytes) {
  gqla_status st = path == GQLA_PATH_GQA ? check_shape_expanded(shape) : check_shape(shape);
  if (st != GQLA_OK) return st;
  if (!plan || !qa || !qr || !out || !ws) return GQLA_ERR_NULL;
  if (!same_shape(plan->shape, *shape) || plan->path != path) return GQLA_ERR_PLAN;
  if (!aligned16(qa) || !aligned16(qr) || !aligned16(out) || !aligned16(ws) || (lse && (reinterpret_cast<uintptr_t>(lse) & 3u)))
    return GQLA_ERR_ALIGN;
  int32_t max_len = 0;
  for (int32_t L : plan->lens) max_len = std::max(max_len, L);
  st = check_cache(shape, cache, plan->page_size, max_len);
  if (st != GQLA_OK) return st;
  if (ws_bytes < plan->ws.total || plan->uploaded_ws != ws) return GQLA_ERR_WORKSPACE;
  return GQLA_OK;
}

// Measurement aid (gqla_time_next_decode_kernel): events that the next decode call of this thread records around its
// split-L decode kernel.
thread_local hipEvent_t t_ev_begin = nullptr, t_ev_end = nullptr;

struct KernelTimer {  // takes the pending pair; record_begin / record_end are no-ops without one
  hipEvent_t e0, e1;
  hipStream_t s;
  explicit KernelTimer(hipStream_t stream) : e0(t_ev_begin), e1(t_ev_end), s(stream) { t_ev_begin = t_ev_end = nullptr; }
  hipError_t begin() const { return e0 ? hipEventRecord(e0, s) : hipSuccess; }
  hipError_t end() const { return e1 ? hipEventRecord(e1, s) : hipSuccess; }
};

CacheView view_of(const gqla_cache* c) {
  CacheView v;
  v.pool = c->pool;
  v.page_table = c->page_table;
  v.page_size = c->page_size;
  v.max_pages = c->max_pages;
  v.num_pages = c->num_pages;
  v.groups = c->groups;
  return v;
}

DecodeArgs decode_args(const gqla_shape* s, const gqla_plan* plan, const void* qa, const void* qr, const gqla_cache* c,
                       void* ws) {
  DecodeArgs a;
  a.q_a = qa;
  a.q_r = qr;
  a.cache = view_of(c);
  a.chunks = reinterpret_cast<const ChunkEntry*>(static_cast<char*>(ws) + plan->ws.table_off);
  a.n_chunks = (int32_t)plan->chunks.size();
  a.part_o = static_cast<char*>(ws) + plan->ws.part_o_off;
  a.part_lse = reinterpret_cast<float*>(static_cast<char*>(ws) + plan->ws.part_lse_off);
  a.B = s->batch;
  a.h_q = s->h_q;
  a.g = s->g;
  a.G = s->h_q / s->g;
  a.d_h = s->d_h;
  a.d_v = value_dim(s);
  a.r_kv = s->r_kv;
  a.d_r = s->d_r;
  a.s_q = s->s_q;
  a.M = s->s_q * s->h_q;
  a.num_cus = plan->num_cus;
  a.scale_log2e = resolved_scale(s) * 1.4426950408889634f;
  return a;
}

CombineArgs combine_args(const gqla_shape* s, const gqla_plan* plan, void* ws, const void* w_uv, void* out, float* lse) {
  CombineArgs c;
  c.part_o = static_cast<char*>(ws) + plan->ws.part_o_off;
  c.part_lse = reinterpret_cast<const float*>(static_cast<char*>(ws) + plan->ws.part_lse_off);
  c.first_slot = reinterpret_cast<const int32_t*>(static_cast<char*>(ws) + plan->ws.first_slot_off);
  c.w_uv = w_uv;
  c.out = out;
  c.lse = lse;
  c.B = s->batch;
  c.h_q = s->h_q;
  c.g = s->g;
  c.G = s->h_q / s->g;
  c.d_h = s->d_h;
  c.r_kv = s->r_kv;
  c.s_q = s->s_q;
  c.M = s->s_q * s->h_q;
  return c;
}

}  // namespace

extern "C" {

gqla_status gqla_plan_create(const gqla_shape* shape, const int32_t* seq_lens_host, int32_t page_size, int32_t num_cus,
                             int32_t path, int32_t chunk_pages_override, gqla_plan** out) {
  if (!out) return GQLA_ERR_NULL;
  *out = nullptr;
  gqla_status st = check_shape(shape);
  if (st != GQLA_OK) return st;
  if (!seq_lens_host && shape->batch > 0) return GQLA_ERR_NULL;
  if (path != GQLA_PATH_ABSORB && path != GQLA_PATH_GQA) return GQLA_ERR_PLAN;
  if (path == GQLA_PATH_GQA && check_shape_expanded(shape) != GQLA_OK) return GQLA_ERR_SHAPE;
  if (num_cus <= 0 || chunk_pages_override < 0) return GQLA_ERR_SHAPE;
  st = check_page_size(shape, page_size);
  if (st != GQLA_OK) return st;
  if (path == GQLA_PATH_GQA && shape->dtype == GQLA_BF16 && (int64_t)(shape->h_q / shape->g) * shape->s_q > 32 * 64)
    return GQLA_ERR_SHAPE;
  for (int32_t b = 0; b < shape->batch; ++b)
    if (seq_lens_host[b] < shape->s_q) return GQLA_ERR_SEQLEN;

  gqla_plan* p = new (std::nothrow) gqla_plan();
  if (!p) return GQLA_ERR_DEVICE;
  p->shape = *shape;
  p->path = path;
  p->page_size = page_size;
  p->num_cus = num_cus;
  p->uploaded_ws = nullptr;
  p->lens.assign(seq_lens_host, seq_lens_host + shape->batch);

  std::vector<int32_t> npages(shape->batch);
  int32_t max_np = 1;
  for (int32_t b = 0; b < shape->batch; ++b) {
    npages[b] = (int32_t)ceil_div(p->lens[b], page_size);
    max_np = std::max(max_np, npages[b]);
  }
  int32_t cp = chunk_pages_override;
  if (cp == 0) cp = choose_chunk_pages(npages, *shape, num_cus, path);
  p->chunk_pages = cp;
  p->first_slot.resize(shape->batch + 1);
  for (int32_t b = 0; b < shape->batch; ++b) {
    p->first_slot[b] = (int32_t)p->chunks.size();
    const int32_t n_b = (int32_t)ceil_div(npages[b], cp);
    const int32_t per = (int32_t)ceil_div(npages[b], n_b);
    for (int32_t k = 0; (int64_t)k * per < npages[b]; ++k) {
      ChunkEntry e;
      e.b = b;
      e.tok_begin = k * per * page_size;
      e.tok_end = (int32_t)std::min<int64_t>((int64_t)(k + 1) * per * page_size, p->lens[b]);
      e.L = p->lens[b];
      p->chunks.push_back(e);
    }
  }
  p->first_slot[shape->batch] = (int32_t)p->chunks.size();
  p->ws = make_layout(*p);
  *out = p;
  return GQLA_OK;
}

void gqla_plan_destroy(gqla_plan* plan) { delete plan; }

int32_t gqla_plan_num_chunks(const gqla_plan* plan) { return plan ? (int32_t)plan->chunks.size() : 0; }
int32_t gqla_plan_chunk_pages(const gqla_plan* plan) { return plan ? plan->chunk_pages : 0; }

gqla_status gqla_plan_export(const gqla_plan* plan, int32_t* triples, int32_t* first_slot, int32_t* n) {
  if (!plan || !n) return GQLA_ERR_NULL;
  const int32_t have = (int32_t)plan->chunks.size();
  if (triples) {
    const int32_t m = std::min(*n, have);
    for (int32_t k = 0; k < m; ++k) {
      triples[3 * k] = plan->chunks[k].b;
      triples[3 * k + 1] = plan->chunks[k].tok_begin;
      triples[3 * k + 2] = plan->chunks[k].tok_end;
    }
  }
  if (first_slot)
    for (int32_t b = 0; b < plan->shape.batch; ++b) first_slot[b] = plan->first_slot[b];
  *n = have;
  return GQLA_OK;
}

size_t gqla_plan_workspace_bytes(const gqla_plan* plan) { return plan ? plan->ws.total : 0; }

gqla_status gqla_plan_upload(gqla_plan* plan, void* ws, size_t ws_bytes, void* stream) {
  if (!plan || !ws) return GQLA_ERR_NULL;
  if (!aligned16(ws)) return GQLA_ERR_ALIGN;
  if (ws_bytes < plan->ws.total) return GQLA_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  char* base = static_cast<char*>(ws);
  if (!plan->chunks.empty()) {
    if (hipMemcpyAsync(base + plan->ws.table_off, plan->chunks.data(), plan->chunks.size() * sizeof(ChunkEntry),
                       hipMemcpyHostToDevice, s) != hipSuccess)
      return GQLA_ERR_DEVICE;
  }
  if (hipMemcpyAsync(base + plan->ws.first_slot_off, plan->first_slot.data(), plan->first_slot.size() * sizeof(int32_t),
                     hipMemcpyHostToDevice, s) != hipSuccess)
    return GQLA_ERR_DEVICE;
  plan->uploaded_ws = ws;
  return GQLA_OK;
}

gqla_status gqla_absorb_query(const gqla_shape* shape, const void* q_c, const void* w_uk, void* q_hat, void* stream) {
  gqla_status st = check_shape(shape);
  if (st != GQLA_OK) return st;
  if (!q_c || !w_uk || !q_hat) return GQLA_ERR_NULL;
  if (!aligned16(q_c) || !aligned16(w_uk) || !aligned16(q_hat)) return GQLA_ERR_ALIGN;
  if (shape->batch == 0) return GQLA_OK;
  AbsorbQueryArgs a;
  a.q_c = q_c;
  a.w_uk = w_uk;
  a.q_hat = q_hat;
  a.rows = shape->batch * shape->s_q;
  a.h_q = shape->h_q;
  a.g = shape->g;
  a.G = shape->h_q / shape->g;
  a.d_h = shape->d_h;
  a.r_kv = shape->r_kv;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = shape->dtype == GQLA_BF16 ? launch_absorb_query_bf16(a, s) : launch_absorb_query_f32(a, s);
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

gqla_status gqla_decode_absorb(const gqla_shape* shape, const gqla_plan* plan, const void* q_hat, const void* q_r,
                               const gqla_cache* latent, const void* w_uv, void* out, float* lse, void* ws,
                               size_t ws_bytes, void* stream) {
  gqla_status st = check_decode_common(shape, plan, GQLA_PATH_ABSORB, latent, q_hat, q_r, out, lse, ws, ws_bytes);
  if (st != GQLA_OK) return st;
  if (!w_uv) return GQLA_ERR_NULL;
  if (!aligned16(w_uv)) return GQLA_ERR_ALIGN;
  if (shape->batch == 0) return GQLA_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const DecodeArgs a = decode_args(shape, plan, q_hat, q_r, latent, ws);
  CombineArgs c = combine_args(shape, plan, ws, w_uv, out, lse);
  c.d_h = value_dim(shape);  // the projection's output (and W_UV's columns) are value dims
  const KernelTimer timer(s);
  hipError_t e = timer.begin();
  if (e != hipSuccess) return GQLA_ERR_DEVICE;
  if (shape->dtype == GQLA_BF16) {
    e = launch_decode_absorb_bf16(a, s);
    if (e == hipSuccess) e = timer.end();
    if (e == hipSuccess) e = launch_combine_project_bf16(c, s);
  } else {
    e = launch_decode_absorb_f32(a, s);
    if (e == hipSuccess) e = timer.end();
    if (e == hipSuccess) e = launch_combine_project_f32(c, s);
  }
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

size_t gqla_expand_workspace_bytes(const gqla_shape* shape, int32_t group_count) {
  if (!shape || check_shape_expanded(shape) != GQLA_OK || shape->dtype != GQLA_BF16 || group_count <= 0) return 0;
  return (size_t)group_count * shape->r_kv * (shape->d_h + value_dim(shape)) * 2;  // both weight slices in fragment order, bf16
}

namespace {
// tail = 0: every token of every sequence; tail > 0: the last `tail` positions only
gqla_status expand_impl(const gqla_shape* shape, const gqla_cache* latent, const void* w_uk, const void* w_uv,
                        int32_t group_begin, int32_t group_count, const gqla_cache* expanded, int32_t tail, void* ws,
                        size_t ws_bytes, void* stream, bool fp8 = false, float k_scale = 1.f, float v_scale = 1.f,
                        bool weights_packed = false) {
  gqla_status st = fp8 ? check_shape_equal_dims(shape) : check_shape_expanded(shape);
  if (st != GQLA_OK) return st;
  if (!latent || !expanded || !latent->pool || !expanded->pool || !latent->seq_lens) return GQLA_ERR_NULL;
  if (!weights_packed && (!w_uk || !w_uv)) return GQLA_ERR_NULL;
  if (!aligned16(w_uk) || !aligned16(w_uv) || !aligned16(latent->pool) || !aligned16(expanded->pool)) return GQLA_ERR_ALIGN;
  if (group_begin < 0 || group_count <= 0 || group_begin + group_count > shape->g || expanded->groups != group_count)
    return GQLA_ERR_SHAPE;
  st = check_page_size(shape, latent->page_size);
  if (st != GQLA_OK) return st;
  if (latent->page_size != expanded->page_size || latent->max_pages != expanded->max_pages || latent->max_pages <= 0 ||
      latent->num_pages <= 0 || expanded->num_pages <= 0)
    return GQLA_ERR_PAGE;
  if (!latent->page_table && (int64_t)latent->num_pages < (int64_t)shape->batch * latent->max_pages) return GQLA_ERR_PAGE;
  if (!expanded->page_table && (int64_t)expanded->num_pages < (int64_t)shape->batch * expanded->max_pages) return GQLA_ERR_PAGE;
  if (shape->dtype == GQLA_BF16) {
    if (!ws || ws_bytes < gqla_expand_workspace_bytes(shape, group_count)) return GQLA_ERR_WORKSPACE;
    if (!aligned16(ws)) return GQLA_ERR_ALIGN;
  }
  if (shape->batch == 0) return GQLA_OK;
  ExpandArgs a;
  a.latent = view_of(latent);
  a.expanded = view_of(expanded);
  a.seq_lens = latent->seq_lens;
  a.w_uk = w_uk;
  a.w_uv = w_uv;
  a.B = shape->batch;
  a.g = shape->g;
  a.d_h = shape->d_h;
  a.d_v = value_dim(shape);
  a.r_kv = shape->r_kv;
  a.d_r = shape->d_r;
  a.group_begin = group_begin;
  a.group_count = group_count;
  a.tail = tail;
  a.weights = weights_packed ? 2 : 0;
  a.k_inv_scale = 1.0f / k_scale;
  a.v_inv_scale = 1.0f / v_scale;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (fp8) e = tail > 0 ? launch_expand_tail_fp8(a, ws, s) : launch_expand_fp8(a, ws, s);
  else if (tail > 0) e = shape->dtype == GQLA_BF16 ? launch_expand_tail_bf16(a, ws, s) : launch_expand_tail_f32(a, s);
  else e = shape->dtype == GQLA_BF16 ? launch_expand_bf16(a, ws, s) : launch_expand_f32(a, s);
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}
}  // namespace

gqla_status gqla_expand_cache(const gqla_shape* shape, const gqla_cache* latent, const void* w_uk, const void* w_uv,
                              int32_t group_begin, int32_t group_count, const gqla_cache* expanded, void* ws,
                              size_t ws_bytes, void* stream) {
  return expand_impl(shape, latent, w_uk, w_uv, group_begin, group_count, expanded, 0, ws, ws_bytes, stream);
}

gqla_status gqla_expand_cache_tail(const gqla_shape* shape, const gqla_cache* latent, const void* w_uk, const void* w_uv,
                                   int32_t group_begin, int32_t group_count, const gqla_cache* expanded,
                                   int32_t tail_tokens, void* ws, size_t ws_bytes, void* stream) {
  if (latent && (tail_tokens < 1 || tail_tokens > latent->page_size)) return GQLA_ERR_SHAPE;
  return expand_impl(shape, latent, w_uk, w_uv, group_begin, group_count, expanded, tail_tokens, ws, ws_bytes, stream);
}

// ---- the weights of a group slice repacked once, the step's expansion from the repacked copy ---------------------------------
gqla_status gqla_pack_expand_weights(const gqla_shape* shape, const void* w_uk, const void* w_uv, int32_t group_begin,
                                     int32_t group_count, void* packed, size_t packed_bytes, void* stream) {
  gqla_status st = check_shape_expanded(shape);
  if (st != GQLA_OK) return st;
  if (shape->dtype != GQLA_BF16) return GQLA_ERR_DTYPE;  // the fp32 kernels read the weights as they are
  if (!w_uk || !w_uv || !packed) return GQLA_ERR_NULL;
  if (!aligned16(w_uk) || !aligned16(w_uv) || !aligned16(packed)) return GQLA_ERR_ALIGN;
  if (group_begin < 0 || group_count <= 0 || group_begin + group_count > shape->g) return GQLA_ERR_SHAPE;
  if (packed_bytes < gqla_expand_workspace_bytes(shape, group_count)) return GQLA_ERR_WORKSPACE;
  ExpandArgs a = {};
  a.w_uk = w_uk;
  a.w_uv = w_uv;
  a.B = 0;
  a.g = shape->g;
  a.d_h = shape->d_h;
  a.d_v = value_dim(shape);
  a.r_kv = shape->r_kv;
  a.d_r = shape->d_r;
  a.group_begin = group_begin;
  a.group_count = group_count;
  a.tail = 1;
  a.weights = 1;
  const hipError_t e = launch_expand_tail_bf16(a, packed, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

gqla_status gqla_expand_cache_tail_packed(const gqla_shape* shape, const gqla_cache* latent, const void* packed,
                                          size_t packed_bytes, int32_t group_count, const gqla_cache* expanded,
                                          int32_t tail_tokens, void* stream) {
  if (shape && shape->dtype != GQLA_BF16) return check_shape(shape) == GQLA_OK ? GQLA_ERR_DTYPE : check_shape(shape);
  if (latent && (tail_tokens < 1 || tail_tokens > latent->page_size)) return GQLA_ERR_SHAPE;
  // (the slice's first group does not matter any more: the repacked copy holds the slice's groups from 0)
  return expand_impl(shape, latent, nullptr, nullptr, 0, group_count, expanded, tail_tokens, const_cast<void*>(packed), packed_bytes,
                     stream, false, 1.f, 1.f, true);
}

// ---- the variant for callers that cannot allocate: scratch in a file-scope device array ---------------------------------
// Every GPU the library runs on holds its own copy of this array at its own address until the process ends.  In host
// code the array's NAME is only a handle for the runtime's symbol lookup, not a device address: the address is looked up
// once per device (hipGetSymbolAddress, with that device current) and only that pointer is ever handed to a kernel.
namespace {
constexpr size_t kStaticScratchBytes = (size_t)2 << 20;  // 2 MiB: both weight slices of 8 groups (r_kv 512, d_h 128) in bf16
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device (looked up on the first call per device), or nullptr with *err set.
void* static_scratch(hipError_t* err) {
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) {
    *err = hipErrorInvalidDevice;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    ptr[dev] = p;
  }
  return ptr[dev];
}
}  // namespace

size_t gqla_expand_cache_tail_static_max_workspace(void) { return kStaticScratchBytes; }

gqla_status gqla_expand_cache_tail_static(const gqla_shape* shape, const gqla_cache* latent, const void* w_uk,
                                          const void* w_uv, int32_t group_begin, int32_t group_count,
                                          const gqla_cache* expanded, int32_t tail_tokens, void* stream) {
  if (latent && (tail_tokens < 1 || tail_tokens > latent->page_size)) return GQLA_ERR_SHAPE;
  const gqla_status st = check_shape_expanded(shape);
  if (st != GQLA_OK) return st;
  if (shape->dtype != GQLA_BF16)  // the fp32 kernels use no scratch at all
    return expand_impl(shape, latent, w_uk, w_uv, group_begin, group_count, expanded, tail_tokens, nullptr, 0, stream);
  if (group_count <= 0) return GQLA_ERR_SHAPE;
  const size_t need = gqla_expand_workspace_bytes(shape, group_count);
  if (need == 0 || need > kStaticScratchBytes) return GQLA_ERR_WORKSPACE;  // slice too large for the fixed scratch
  hipError_t e;
  void* ws = static_scratch(&e);
  if (!ws) return GQLA_ERR_DEVICE;
  return expand_impl(shape, latent, w_uk, w_uv, group_begin, group_count, expanded, tail_tokens, ws, kStaticScratchBytes, stream);
}

gqla_status gqla_expand_cache_tail_fp8(const gqla_shape* shape, const gqla_cache* latent, const void* w_uk, const void* w_uv,
                                       int32_t group_begin, int32_t group_count, const gqla_cache* expanded_fp8,
                                       int32_t tail_tokens, float k_scale, float v_scale, void* ws, size_t ws_bytes,
                                       void* stream) {
  if (shape && shape->dtype != GQLA_BF16) return check_shape(shape) == GQLA_OK ? GQLA_ERR_DTYPE : check_shape(shape);
  if (latent && (tail_tokens < 1 || tail_tokens > latent->page_size)) return GQLA_ERR_SHAPE;
  if (!(k_scale > 0.f) || !(v_scale > 0.f) || !std::isfinite(k_scale) || !std::isfinite(v_scale)) return GQLA_ERR_SHAPE;
  return expand_impl(shape, latent, w_uk, w_uv, group_begin, group_count, expanded_fp8, tail_tokens, ws, ws_bytes, stream, true,
                     k_scale, v_scale);
}

gqla_status gqla_expand_cache_fp8(const gqla_shape* shape, const gqla_cache* latent, const void* w_uk, const void* w_uv,
                                  int32_t group_begin, int32_t group_count, const gqla_cache* expanded_fp8, float k_scale,
                                  float v_scale, void* ws, size_t ws_bytes, void* stream) {
  if (shape && shape->dtype != GQLA_BF16) return check_shape(shape) == GQLA_OK ? GQLA_ERR_DTYPE : check_shape(shape);
  if (!(k_scale > 0.f) || !(v_scale > 0.f) || !std::isfinite(k_scale) || !std::isfinite(v_scale)) return GQLA_ERR_SHAPE;
  return expand_impl(shape, latent, w_uk, w_uv, group_begin, group_count, expanded_fp8, 0, ws, ws_bytes, stream, true, k_scale,
                     v_scale);
}

gqla_status gqla_append_latent(const gqla_shape* shape, const void* rows, const gqla_cache* latent, void* stream) {
  gqla_status st = check_shape(shape);
  if (st != GQLA_OK) return st;
  if (!rows || !latent || !latent->pool || !latent->seq_lens) return GQLA_ERR_NULL;
  if (!aligned16(rows) || !aligned16(latent->pool)) return GQLA_ERR_ALIGN;
  st = check_page_size(shape, latent->page_size);
  if (st != GQLA_OK) return st;
  if (latent->max_pages <= 0 || latent->num_pages <= 0) return GQLA_ERR_PAGE;
  if (!latent->page_table && (int64_t)latent->num_pages < (int64_t)shape->batch * latent->max_pages) return GQLA_ERR_PAGE;
  if (shape->batch == 0) return GQLA_OK;
  AppendArgs a;
  a.rows = rows;
  a.latent = view_of(latent);
  a.seq_lens = latent->seq_lens;
  a.B = shape->batch;
  a.s_q = shape->s_q;
  a.row_bytes = (shape->r_kv + shape->d_r) * (shape->dtype == GQLA_BF16 ? 2 : 4);
  const hipError_t e = launch_append_latent(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

gqla_status gqla_decode_gqa(const gqla_shape* shape, const gqla_plan* plan, const void* q_c, const void* q_r,
                            const gqla_cache* expanded, void* out, float* lse, void* ws, size_t ws_bytes, void* stream) {
  gqla_status st = check_decode_common(shape, plan, GQLA_PATH_GQA, expanded, q_c, q_r, out, lse, ws, ws_bytes);
  if (st != GQLA_OK) return st;
  if (expanded->groups != shape->g) return GQLA_ERR_SHAPE;
  if (shape->batch == 0) return GQLA_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const DecodeArgs a = decode_args(shape, plan, q_c, q_r, expanded, ws);
  CombineArgs c = combine_args(shape, plan, ws, nullptr, out, lse);
  c.d_h = value_dim(shape);  // partials and outputs are value dims
  const KernelTimer timer(s);
  hipError_t e = timer.begin();
  if (e == hipSuccess) e = shape->dtype == GQLA_BF16 ? launch_decode_gqa_bf16(a, s) : launch_decode_gqa_f32(a, s);
  if (e == hipSuccess) e = timer.end();
  if (e == hipSuccess) e = shape->dtype == GQLA_BF16 ? launch_combine_gqa_bf16(c, s) : launch_combine_f32(c, s);
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

gqla_status gqla_rope_step(const gqla_shape* shape, const int32_t* seq_lens, float rope_base, void* q_r, void* rows,
                           void* stream) {
  gqla_status st = check_shape(shape);
  if (st != GQLA_OK) return st;
  if (!seq_lens || (!q_r && !rows)) return GQLA_ERR_NULL;
  if ((q_r && !aligned16(q_r)) || (rows && !aligned16(rows))) return GQLA_ERR_ALIGN;
  if (!(rope_base > 1.0f) || !std::isfinite(rope_base) || shape->d_r % 2 || shape->d_r > 512 || shape->r_kv % 2) return GQLA_ERR_SHAPE;
  if (shape->batch == 0) return GQLA_OK;
  RopeArgs a;
  a.q_r = q_r;
  a.rows = rows;
  a.seq_lens = seq_lens;
  a.log2_base = std::log2((double)rope_base);
  a.B = shape->batch;
  a.s_q = shape->s_q;
  a.h_q = shape->h_q;
  a.d_r = shape->d_r;
  a.r_kv = shape->r_kv;
  a.row_elems = shape->r_kv + shape->d_r;
  const hipError_t e = launch_rope_step(a, shape->dtype == GQLA_BF16, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

size_t gqla_output_projection_workspace_bytes(const gqla_shape* shape, int32_t d_model) {
  if (check_shape(shape) != GQLA_OK || d_model <= 0 || shape->dtype != GQLA_BF16) return 0;
  const int64_t M = (int64_t)shape->batch * shape->s_q, K = (int64_t)shape->h_q * value_dim(shape);
  if (M == 0 || d_model % 128 || K % 256 || K > (1 << 24)) return 0;
  int krange = 0;
  const int ksplit = out_proj_split((int)M, (int)K, d_model, &krange);
  return ksplit > 1 ? (size_t)ksplit * M * d_model * sizeof(float) : 0;
}

gqla_status gqla_output_projection(const gqla_shape* shape, int32_t d_model, const void* o, const void* w_o, void* y,
                                   void* ws, size_t ws_bytes, void* stream) {
  gqla_status st = check_shape(shape);
  if (st != GQLA_OK) return st;
  if (!o || !w_o || !y) return GQLA_ERR_NULL;
  if (!aligned16(o) || !aligned16(w_o) || !aligned16(y) || (ws && !aligned16(ws))) return GQLA_ERR_ALIGN;
  if (d_model <= 0) return GQLA_ERR_SHAPE;
  const int64_t M = (int64_t)shape->batch * shape->s_q, K = (int64_t)shape->h_q * value_dim(shape);
  if (M > INT32_MAX || K > INT32_MAX) return GQLA_ERR_SHAPE;
  if (M == 0) return GQLA_OK;
  OutProjArgs a;
  a.o = o;
  a.w_o = w_o;
  a.y = y;
  a.partial = nullptr;
  a.M = (int32_t)M;
  a.K = (int32_t)K;
  a.D = d_model;
  a.ksplit = 1;
  a.krange = (int32_t)K;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (shape->dtype != GQLA_BF16) return launch_out_proj_f32(a, s) == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
  if (d_model % 128 || K % 256 || K > (1 << 24)) return GQLA_ERR_SHAPE;   // the kernel's row offsets inside a tile are 32-bit
  a.ksplit = out_proj_split(a.M, a.K, a.D, &a.krange);
  if (a.ksplit > 1) {
    if (!ws) return GQLA_ERR_NULL;
    if (ws_bytes < (size_t)a.ksplit * M * d_model * sizeof(float)) return GQLA_ERR_WORKSPACE;
    a.partial = static_cast<float*>(ws);
  }
  return launch_out_proj_bf16(a, s) == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

gqla_status gqla_left_inverse(const gqla_shape* shape, const float* w_uk_host, float* w_inv_host) {
  gqla_status st = check_shape(shape);
  if (st != GQLA_OK) return st;
  if (!w_uk_host || !w_inv_host) return GQLA_ERR_NULL;
  const int g = shape->g, r = shape->r_kv, d = shape->d_h;
  const int K = g * d;
  if (K < r) return GQLA_ERR_SHAPE;  // the stacked key up-projection cannot have full column rank
  // Gram matrix G = A^T A = sum_j W_UK[j] W_UK[j]^T (r x r), in double
  std::vector<double> G((size_t)r * r, 0.0);
  for (int j = 0; j < g; ++j) {
    const float* w = w_uk_host + (size_t)j * r * d;
    for (int x = 0; x < r; ++x)
      for (int y = 0; y <= x; ++y) {
        double acc = 0.0;
        for (int k = 0; k < d; ++k) acc += (double)w[(size_t)x * d + k] * (double)w[(size_t)y * d + k];
        G[(size_t)x * r + y] += acc;
      }
  }
  // Cholesky G = C C^T (lower triangle in place)
  for (int x = 0; x < r; ++x) {
    for (int y = 0; y <= x; ++y) {
      const double diag = G[(size_t)x * r + y];
      double acc = diag;
      for (int k = 0; k < y; ++k) acc -= G[(size_t)x * r + k] * G[(size_t)y * r + k];
      if (x == y) {
        if (!(acc > 1e-12 * diag)) return GQLA_ERR_SHAPE;  // rank deficient up to the rounding of the Gram matrix
        G[(size_t)x * r + x] = std::sqrt(acc);
      } else {
        G[(size_t)x * r + y] = acc / G[(size_t)y * r + y];
      }
    }
  }
  // columns of A^T are the rows of A: column (j, k) of A^T is W_UK[j][:, k]; solve G z = that column
  std::vector<double> z(r);
  for (int j = 0; j < g; ++j)
    for (int k = 0; k < d; ++k) {
      const float* w = w_uk_host + (size_t)j * r * d + k;
      for (int x = 0; x < r; ++x) {  // forward: C u = a
        double acc = (double)w[(size_t)x * d];
        for (int y = 0; y < x; ++y) acc -= G[(size_t)x * r + y] * z[y];
        z[x] = acc / G[(size_t)x * r + x];
      }
      for (int x = r - 1; x >= 0; --x) {  // backward: C^T z = u
        double acc = z[x];
        for (int y = x + 1; y < r; ++y) acc -= G[(size_t)y * r + x] * z[y];
        z[x] = acc / G[(size_t)x * r + x];
      }
      for (int x = 0; x < r; ++x) w_inv_host[(size_t)x * K + (size_t)j * d + k] = (float)z[x];
    }
  return GQLA_OK;
}

gqla_status gqla_compress_cache(const gqla_shape* shape, const gqla_cache* expanded, const void* w_inv,
                                const gqla_cache* latent, void* stream) {
  gqla_status st = check_shape_expanded(shape);
  if (st != GQLA_OK) return st;
  if (!expanded || !latent || !w_inv || !expanded->pool || !latent->pool || !expanded->seq_lens) return GQLA_ERR_NULL;
  if (!aligned16(w_inv) || !aligned16(expanded->pool) || !aligned16(latent->pool)) return GQLA_ERR_ALIGN;
  if (expanded->groups != shape->g || shape->g * shape->d_h < shape->r_kv) return GQLA_ERR_SHAPE;
  st = check_page_size(shape, expanded->page_size);
  if (st != GQLA_OK) return st;
  if (latent->page_size != expanded->page_size || latent->max_pages != expanded->max_pages || latent->max_pages <= 0 ||
      latent->num_pages <= 0 || expanded->num_pages <= 0)
    return GQLA_ERR_PAGE;
  if (!latent->page_table && (int64_t)latent->num_pages < (int64_t)shape->batch * latent->max_pages) return GQLA_ERR_PAGE;
  if (!expanded->page_table && (int64_t)expanded->num_pages < (int64_t)shape->batch * expanded->max_pages) return GQLA_ERR_PAGE;
  if (shape->batch == 0) return GQLA_OK;
  CompressArgs a;
  a.expanded = view_of(expanded);
  a.latent = view_of(latent);
  a.seq_lens = expanded->seq_lens;
  a.w_inv = w_inv;
  a.B = shape->batch;
  a.g = shape->g;
  a.d_h = shape->d_h;
  a.d_v = value_dim(shape);
  a.r_kv = shape->r_kv;
  a.d_r = shape->d_r;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const hipError_t e = shape->dtype == GQLA_BF16 ? launch_compress_bf16(a, s) : launch_compress_f32(a, s);
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

gqla_status gqla_quantize_expanded(const gqla_shape* shape, const gqla_cache* expanded, const gqla_cache* expanded_fp8,
                                   float k_scale, float v_scale, void* stream) {
  gqla_status st = check_shape_equal_dims(shape);
  if (st != GQLA_OK) return st;
  if (shape->dtype != GQLA_BF16) return GQLA_ERR_DTYPE;
  if (!expanded || !expanded_fp8 || !expanded->pool || !expanded_fp8->pool || !expanded->seq_lens) return GQLA_ERR_NULL;
  if (!aligned16(expanded->pool) || !aligned16(expanded_fp8->pool)) return GQLA_ERR_ALIGN;
  if (!(k_scale > 0.f) || !(v_scale > 0.f) || !std::isfinite(k_scale) || !std::isfinite(v_scale)) return GQLA_ERR_SHAPE;
  if (expanded->groups <= 0 || expanded->groups > shape->g || expanded->groups != expanded_fp8->groups) return GQLA_ERR_SHAPE;
  st = check_page_size(shape, expanded->page_size);
  if (st != GQLA_OK) return st;
  if (expanded->page_size != expanded_fp8->page_size || expanded->max_pages != expanded_fp8->max_pages ||
      expanded->max_pages <= 0 || expanded->num_pages <= 0 || expanded_fp8->num_pages <= 0)
    return GQLA_ERR_PAGE;
  if (!expanded->page_table && (int64_t)expanded->num_pages < (int64_t)shape->batch * expanded->max_pages) return GQLA_ERR_PAGE;
  if (!expanded_fp8->page_table && (int64_t)expanded_fp8->num_pages < (int64_t)shape->batch * expanded_fp8->max_pages)
    return GQLA_ERR_PAGE;
  if (shape->batch == 0) return GQLA_OK;
  QuantizeArgs a;
  a.src = view_of(expanded);
  a.dst = view_of(expanded_fp8);
  a.seq_lens = expanded->seq_lens;
  a.B = shape->batch;
  a.k_inv_scale = 1.0f / k_scale;
  a.v_inv_scale = 1.0f / v_scale;
  const hipError_t e = launch_quantize_expanded(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

gqla_status gqla_decode_gqa_fp8(const gqla_shape* shape, const gqla_plan* plan, const void* q_c, const void* q_r,
                                const gqla_cache* expanded_fp8, float k_scale, float v_scale, void* out, float* lse,
                                void* ws, size_t ws_bytes, void* stream) {
  gqla_status st = check_shape_equal_dims(shape);
  if (st != GQLA_OK) return st;
  if (shape->dtype != GQLA_BF16) return GQLA_ERR_DTYPE;
  if (!(k_scale > 0.f) || !(v_scale > 0.f) || !std::isfinite(k_scale) || !std::isfinite(v_scale)) return GQLA_ERR_SHAPE;
  st = check_decode_common(shape, plan, GQLA_PATH_GQA, expanded_fp8, q_c, q_r, out, lse, ws, ws_bytes);
  if (st != GQLA_OK) return st;
  if (expanded_fp8->groups != shape->g) return GQLA_ERR_SHAPE;
  if (shape->batch == 0) return GQLA_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const DecodeArgs a = decode_args(shape, plan, q_c, q_r, expanded_fp8, ws);
  const CombineArgs c = combine_args(shape, plan, ws, nullptr, out, lse);
  const KernelTimer timer(s);
  hipError_t e = timer.begin();
  if (e == hipSuccess) e = launch_decode_gqa_fp8(a, k_scale, v_scale, s);
  if (e == hipSuccess) e = timer.end();
  if (e == hipSuccess) e = launch_combine_gqa_bf16(c, s);
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

gqla_status gqla_quantize_latent(const gqla_shape* shape, const gqla_cache* latent, const gqla_cache* latent_fp8,
                                 float c_scale, void* stream) {
  gqla_status st = check_shape(shape);
  if (st != GQLA_OK) return st;
  if (shape->dtype != GQLA_BF16) return GQLA_ERR_DTYPE;
  if (!latent || !latent_fp8 || !latent->pool || !latent_fp8->pool || !latent->seq_lens) return GQLA_ERR_NULL;
  if (!aligned16(latent->pool) || !aligned16(latent_fp8->pool)) return GQLA_ERR_ALIGN;
  if (!(c_scale > 0.f) || !std::isfinite(c_scale)) return GQLA_ERR_SHAPE;
  st = check_page_size(shape, latent->page_size);
  if (st != GQLA_OK) return st;
  if (latent->page_size != latent_fp8->page_size || latent->max_pages != latent_fp8->max_pages || latent->max_pages <= 0 ||
      latent->num_pages <= 0 || latent_fp8->num_pages <= 0)
    return GQLA_ERR_PAGE;
  if (!latent->page_table && (int64_t)latent->num_pages < (int64_t)shape->batch * latent->max_pages) return GQLA_ERR_PAGE;
  if (!latent_fp8->page_table && (int64_t)latent_fp8->num_pages < (int64_t)shape->batch * latent_fp8->max_pages)
    return GQLA_ERR_PAGE;
  if (shape->batch == 0) return GQLA_OK;
  QuantizeArgs a;
  a.src = view_of(latent);
  a.dst = view_of(latent_fp8);
  a.seq_lens = latent->seq_lens;
  a.B = shape->batch;
  a.k_inv_scale = 1.0f / c_scale;
  a.v_inv_scale = a.k_inv_scale;
  const hipError_t e = launch_quantize_latent(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

gqla_status gqla_decode_absorb_fp8(const gqla_shape* shape, const gqla_plan* plan, const void* q_hat, const void* q_r,
                                   const gqla_cache* latent_fp8, float c_scale, const void* w_uv, void* out, float* lse,
                                   void* ws, size_t ws_bytes, void* stream) {
  gqla_status st = check_shape(shape);
  if (st != GQLA_OK) return st;
  if (shape->dtype != GQLA_BF16) return GQLA_ERR_DTYPE;
  if (!(c_scale > 0.f) || !std::isfinite(c_scale)) return GQLA_ERR_SHAPE;
  st = check_decode_common(shape, plan, GQLA_PATH_ABSORB, latent_fp8, q_hat, q_r, out, lse, ws, ws_bytes);
  if (st != GQLA_OK) return st;
  if (!w_uv) return GQLA_ERR_NULL;
  if (!aligned16(w_uv)) return GQLA_ERR_ALIGN;
  if (shape->batch == 0) return GQLA_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const DecodeArgs a = decode_args(shape, plan, q_hat, q_r, latent_fp8, ws);
  CombineArgs c = combine_args(shape, plan, ws, w_uv, out, lse);
  c.d_h = value_dim(shape);
  const KernelTimer timer(s);
  hipError_t e = timer.begin();
  if (e == hipSuccess) e = launch_decode_absorb_fp8(a, c_scale, s);
  if (e == hipSuccess) e = timer.end();
  if (e == hipSuccess) e = launch_combine_project_bf16(c, s);
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

int64_t gqla_latent_fp8_bytes_per_token(int32_t r_kv, int32_t d_r) { return (int64_t)r_kv + 2ll * d_r; }
int64_t gqla_expanded_fp8_bytes_per_token(int32_t groups, int32_t d_h, int32_t d_r) { return 2ll * groups * d_h + 2ll * d_r; }
int64_t gqla_latent_elems_per_token(int32_t r_kv, int32_t d_r) { return (int64_t)r_kv + d_r; }
int64_t gqla_expanded_elems_per_token(int32_t groups, int32_t d_h, int32_t d_r) { return 2ll * groups * d_h + d_r; }
int64_t gqla_expanded_elems_per_token_dv(int32_t groups, int32_t d_h, int32_t d_v, int32_t d_r) {
  return (int64_t)groups * ((int64_t)d_h + d_v) + d_r;
}
int64_t gqla_expanded_k_offset_dv(int64_t page, int32_t j, int32_t slot, int32_t d, int32_t P, int32_t groups, int32_t d_h, int32_t d_v, int32_t d_r) {
  return page * P * gqla_expanded_elems_per_token_dv(groups, d_h, d_v, d_r) + (((int64_t)j * (d_h / 8) + d / 8) * P + slot) * 8 + d % 8;
}
int64_t gqla_expanded_v_offset_dv(int64_t page, int32_t j, int32_t slot, int32_t d, int32_t P, int32_t groups, int32_t d_h, int32_t d_v, int32_t d_r) {
  return page * P * gqla_expanded_elems_per_token_dv(groups, d_h, d_v, d_r) + (int64_t)groups * P * d_h +
         (((int64_t)j * (P / 8) + slot / 8) * d_v + d) * 8 + slot % 8;
}
int64_t gqla_expanded_kr_offset_dv(int64_t page, int32_t slot, int32_t d, int32_t P, int32_t groups, int32_t d_h, int32_t d_v, int32_t d_r) {
  return page * P * gqla_expanded_elems_per_token_dv(groups, d_h, d_v, d_r) + (int64_t)groups * P * ((int64_t)d_h + d_v) +
         ((int64_t)(d / 8) * P + slot) * 8 + d % 8;
}
int64_t gqla_latent_offset(int64_t page, int32_t slot, int32_t col, int32_t page_size, int32_t r_kv, int32_t d_r) {
  return (page * page_size + slot) * ((int64_t)r_kv + d_r) + col;
}
int64_t gqla_expanded_k_offset(int64_t page, int32_t j, int32_t slot, int32_t d, int32_t P, int32_t groups, int32_t d_h, int32_t d_r) {
  return page * P * (2ll * groups * d_h + d_r) + (((int64_t)j * (d_h / 8) + d / 8) * P + slot) * 8 + d % 8;
}
int64_t gqla_expanded_v_offset(int64_t page, int32_t j, int32_t slot, int32_t d, int32_t P, int32_t groups, int32_t d_h, int32_t d_r) {
  return page * P * (2ll * groups * d_h + d_r) + (int64_t)groups * P * d_h + (((int64_t)j * (P / 8) + slot / 8) * d_h + d) * 8 + slot % 8;
}
int64_t gqla_expanded_kr_offset(int64_t page, int32_t slot, int32_t d, int32_t P, int32_t groups, int32_t d_h, int32_t d_r) {
  return page * P * (2ll * groups * d_h + d_r) + 2ll * groups * P * d_h + ((int64_t)(d / 8) * P + slot) * 8 + d % 8;
}

gqla_status gqla_estimate_paths(const gqla_shape* shape, int64_t cached_tokens, double hbm_bytes_per_s,
                                double mfma_flops_per_s, gqla_path_estimate* out) {
  if (!out) return GQLA_ERR_NULL;
  gqla_status st = check_shape(shape);
  if (st != GQLA_OK) return st;
  if (cached_tokens < 0 || !(hbm_bytes_per_s > 0.0) || !(mfma_flops_per_s > 0.0)) return GQLA_ERR_SHAPE;
  const double L = (double)cached_tokens, elem = shape->dtype == GQLA_BF16 ? 2.0 : 4.0;
  const double rows = (double)shape->h_q * shape->s_q;
  out->absorb_bytes = L * elem * (shape->r_kv + shape->d_r);
  out->absorb_flops = 2.0 * L * rows * (2.0 * shape->r_kv + shape->d_r);
  out->absorb_intensity = rows * (2.0 * shape->r_kv + shape->d_r) / (elem / 2.0 * (shape->r_kv + shape->d_r));
  const double d_v = value_dim(shape);
  out->gqa_bytes = L * elem * (shape->g * (shape->d_h + d_v) + shape->d_r);
  out->gqa_flops = 2.0 * L * rows * (shape->d_h + d_v + shape->d_r);
  out->gqa_intensity = rows * (shape->d_h + d_v + shape->d_r) / (elem / 2.0 * (shape->g * (shape->d_h + d_v) + shape->d_r));
  const double ta_m = out->absorb_bytes / hbm_bytes_per_s, ta_c = out->absorb_flops / mfma_flops_per_s;
  const double tg_m = out->gqa_bytes / hbm_bytes_per_s, tg_c = out->gqa_flops / mfma_flops_per_s;
  out->absorb_seconds = ta_m > ta_c ? ta_m : ta_c;
  out->gqa_seconds = tg_m > tg_c ? tg_m : tg_c;
  out->ridge = mfma_flops_per_s / hbm_bytes_per_s;
  out->faster_path = out->gqa_seconds < out->absorb_seconds ? GQLA_PATH_GQA : GQLA_PATH_ABSORB;
  return GQLA_OK;
}

gqla_status gqla_select_path(const gqla_shape* shape, int64_t cached_tokens, gqla_path_choice* out) {
  if (!out) return GQLA_ERR_NULL;
  gqla_status st = check_shape_equal_dims(shape);
  if (st != GQLA_OK) return st;
  if (shape->dtype != GQLA_BF16) return GQLA_ERR_DTYPE;
  if (cached_tokens < 0) return GQLA_ERR_SHAPE;
  gqla_path_estimate e;
  st = gqla_estimate_paths(shape, cached_tokens, 1.0, 1.0, &e);  // only its byte and FLOP counts are used
  if (st != GQLA_OK) return st;
  const double row_blocks = (double)(((shape->h_q / shape->g) * shape->s_q + 31) / 32);
  // absorb, throughput form: the rates the kernel sustains when every compute unit has a long chunk
  double ta = 24e-6 + std::max(e.absorb_bytes / 5.5e12, e.absorb_flops / 1.09e15);
  // absorb, critical path of one workgroup: the split plan of `batch` equal sequences on 64-token pages and 256 compute
  // units gives every workgroup `rounds` chunks of `per` pages; a page costs a workgroup 3.8 us (128 rows, one wave
  // per 32 rows), 3.0 us with 64 rows (two of the four waves have rows), 2.6 us when the chunks are so few that the
  // launch gives every 32 rows a workgroup of their own, and 1.6 us when a sequence has at most 32 rows; a chunk's
  // fixed cost is that of 4 pages.
  if (shape->batch > 0 && cached_tokens > 0) {
    const int64_t np = ceil_div(ceil_div(cached_tokens, shape->batch), 64);
    const int64_t slots = plan_slots(*shape, 256, GQLA_PATH_ABSORB);
    const int64_t cp = choose_chunk_pages(std::vector<int32_t>((size_t)shape->batch, (int32_t)np), *shape, 256, GQLA_PATH_ABSORB);
    const int64_t per_seq = ceil_div(np, cp), per = ceil_div(np, per_seq), chunks = shape->batch * per_seq;
    const int64_t M = (int64_t)shape->h_q * shape->s_q;
    const double page_s = M <= 32 ? 1.6e-6 : (ceil_div(chunks, 8) * 8 * ceil_div(M, 32) <= 256 ? 2.6e-6 : (M <= 64 ? 3.0e-6 : 3.8e-6));
    ta = std::max(ta, 24e-6 + (double)(ceil_div(chunks, slots) * (per + 4)) * page_s);
  }
  out->absorb_seconds = ta;
  // GQA: a fixed cost plus the cache bytes at the rate the kernel streams them -- 7.0 TB/s from HBM; a cache of up to
  // 200 MB is still in the chip's last-level cache from the previous step and streams at about 10 TB/s.  (A group with
  // 64 query rows costs a few percent more per byte than one with 32: a wave then takes both row blocks.)
  const double gqa_bytes = (1.0 + 0.05 * (row_blocks - 1.0)) * e.gqa_bytes;
  out->gqa_seconds = 26e-6 + std::min(gqa_bytes, 200e6) / 10e12 + std::max(0.0, gqa_bytes - 200e6) / 7.0e12;
  out->faster_path = out->gqa_seconds < out->absorb_seconds ? GQLA_PATH_GQA : GQLA_PATH_ABSORB;
  return GQLA_OK;
}

gqla_status gqla_probe_stream_read(const void* src, size_t bytes, void* sink, int32_t num_cus, void* stream) {
  if (!src || !sink) return GQLA_ERR_NULL;
  if (!aligned16(src)) return GQLA_ERR_ALIGN;
  if (num_cus <= 0 || bytes == 0 || bytes % ((size_t)16 * 1024 * 8 * num_cus)) return GQLA_ERR_SHAPE;
  const hipError_t e = launch_probe_stream_read(src, bytes, static_cast<uint32_t*>(sink), 8 * num_cus, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

gqla_status gqla_probe_mfma_bf16(void* sink, int32_t iters, int32_t num_cus, void* stream) {
  if (!sink) return GQLA_ERR_NULL;
  if (num_cus <= 0 || iters <= 0) return GQLA_ERR_SHAPE;
  const hipError_t e = launch_probe_mfma(static_cast<uint32_t*>(sink), iters, num_cus, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? GQLA_OK : GQLA_ERR_DEVICE;
}

gqla_status gqla_time_next_decode_kernel(void* event_begin, void* event_end) {
  if (!event_begin != !event_end) return GQLA_ERR_NULL;  // both or neither (neither: forget a pending pair)
  t_ev_begin = static_cast<hipEvent_t>(event_begin);
  t_ev_end = static_cast<hipEvent_t>(event_end);
  return GQLA_OK;
}

double gqla_probe_mfma_flops(int32_t iters, int32_t num_cus) {
  return (double)num_cus * 4.0 /* waves */ * 4.0 /* MFMAs per iteration */ * (double)iters * 32768.0;  // 2 * 32 * 32 * 16 each
}

const char* gqla_status_string(int32_t status) {
  switch (status) {
    case GQLA_OK: return "ok";
    case GQLA_ERR_NULL: return "null pointer";
    case GQLA_ERR_SHAPE: return "unsupported or inconsistent shape";
    case GQLA_ERR_DTYPE: return "unsupported dtype";
    case GQLA_ERR_ALIGN: return "pointer not 16-byte aligned";
    case GQLA_ERR_SEQLEN: return "sequence length out of range";
    case GQLA_ERR_PAGE: return "inconsistent page geometry";
    case GQLA_ERR_WORKSPACE: return "workspace too small or plan table not uploaded into it";
    case GQLA_ERR_DEVICE: return "HIP call failed";
    case GQLA_ERR_PLAN: return "plan does not match shape or path";
    default: return "unknown status";
  }
}

}  // extern "C"
