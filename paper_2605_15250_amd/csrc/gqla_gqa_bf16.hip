// GQA-path split-L decode over the expanded cache, bf16 MFMA (paper Sec. 3.1, GQA-path equation).
//
// One wave per (chunk, 32-row block, group).  The expanded page stores K_C, V and k_R as 16-byte vectors
// that are already MFMA operand fragments, so every cache byte goes HBM -> VGPR once, with no LDS staging:
//   S^T[token][row] = K[token][dim] * Q^T[dim][row]        A = cache vectors, B = queries held in registers
//   O^T[dim][row]  += V^T[dim][token] * P^T[token][row]    A = cache vectors, B = probabilities from S^T
// S^T and O^T keep one query row per lane (row = lane % 32), so the online-softmax state is per lane and the
// only cross-lane traffic is between the two half-waves.  Cache vectors are read once, so their loads carry the
// non-temporal hint.  All heads of a group (G * s_q rows) share each
// loaded vector through the MFMA.  The path is bound by HBM bandwidth (intensity 19-39 FLOP/byte, Sec. 4.2.2).
#include "gqla_device.h"
#include "gqla_lds.h"

namespace gqla {

namespace {

constexpr float kRescaleThreshold = 8.f;  // log2 units

// FP8 = true: K_C and V are E4M3 codes (16-byte vectors holding one lane's elements of two consecutive k-steps, see
// the header's format), widened to bf16 in registers right before their MFMAs; the scales enter once per tile (K: on
// the content part of the logits, before the RoPE part is added) and once per chunk (V: on the normalised output).
// Half the bytes per token, the same MFMAs.
__device__ __forceinline__ bf16x8 widen_e4m3(uint32_t w0, uint32_t w1) {
  // one instruction per two codes (v_cvt_scalef32_pk_bf16_fp8 with scale 1): exact, every E4M3 value is a bf16 value;
  // checked on the chip against the fp32 route (v_cvt_pk_f32_fp8, then round to bf16) for all 256 codes in all four
  // byte positions
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, false), b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, true);
  const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, false), d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, true);
  const u32x4 r = {__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, b), __builtin_bit_cast(uint32_t, c), __builtin_bit_cast(uint32_t, d)};
  return __builtin_bit_cast(bf16x8, r);
}

// DH: key dims per head, DV: value dims per head (d_h^V of Sec. 3.2.2).  MAXT: threads per workgroup at most -- 512
// (two waves per SIMD, 256 registers each) for equal dims of 128; the (192, 256) shape keeps 128 more accumulators and
// 28 cache vectors in flight per wave, needs the whole register file of a SIMD and runs with 256.
// RB: 32-row blocks per wave.  A group with more than 32 query rows (G s_q = 64: 32 heads per group with one
// multi-token-prediction head) gives RB = 2: one wave multiplies every loaded cache vector into both blocks' S^T and
// O^T, so that the vector crosses the vector-memory path once (two waves with 32 rows each would both load it; such a
// wave also needs a SIMD's whole register file: MAXT = 256).  Its query fragments (96 registers' worth, the same for
// every tile) live in LDS instead, 24 KB per wave, and are read back one 16-byte vector per MFMA.
// tt (kernel argument): token team.  1: a wave works through its chunk alone.  8 (one group with at most 32 query rows,
// RB = 1): the eight waves of a workgroup share one chunk, wave w taking tiles w, w + 8, ...; their eight partial
// states (m, l, O^T) are merged through LDS, so that one partial per chunk reaches memory instead of eight.
template <int DH, int DV, int DR, bool FP8, int MAXT, int RB>
__global__ void __launch_bounds__(MAXT) decode_gqa_bf16_kernel(DecodeArgs a, int n_items, int row_blocks, int share_kr_arg,
                                                               int tt_arg, float k_scale, float v_scale) {
  constexpr int KS_C = DH / 16;  // k-steps over the content dims
  constexpr int KS_R = DR / 16;  // k-steps over the RoPE dims
  constexpr int MT = DV / 32;    // 32-dim tiles of the output
  static_assert(!FP8 || DH == DV, "the 8-bit page format is written for equal dims");
  constexpr bool CAN_TEAM = RB == 1 && MT == 4;  // the merge below is written (and its LDS sized) for 64 accumulators per lane
  const int tt = CAN_TEAM ? tt_arg : 1;
  const int lane = threadIdx.x & 63;
  const int wpb = __builtin_amdgcn_readfirstlane(blockDim.x >> 6);  // waves per workgroup: 8, or the number of groups when that is 2 or 4
  const int wave_in_wg = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int item = __builtin_amdgcn_readfirstlane(blockIdx.x * (wpb / tt) + wave_in_wg / tt);  // wave-uniform: keep it scalar
  const int tw = wave_in_wg % tt;   // position in the token team
  const int tstep = 32 * tt;        // tokens from one tile of this wave to its next
  if (item >= n_items) return;      // (a whole token team leaves together)
  const int j = item % a.g;
  const int rb = (item / a.g) % row_blocks;
  const int chunk = item / (a.g * row_blocks);
  const ChunkEntry ce = a.chunks[chunk];
  const int n = lane & 31, h = lane >> 5;

  // query rows of this lane, one per row block x: rho in [0, G*s_q), rho = t*G + head-in-group
  constexpr bool QLDS = RB > 1;  // query fragments in LDS (dynamic shared memory: RB * (KS_C + KS_R) KB per wave)
  extern __shared__ __attribute__((aligned(16))) char dyn_lds[];  // RB > 1: query fragments; tt > 1: the merge buffers
  char* const q_lds = dyn_lds + (threadIdx.x >> 6) * (RB * (KS_C + KS_R) * 1024) + lane * 16;
  bool row_ok[RB];
  int t_of[RB], head_of[RB], vis_end[RB];
  bf16x8 qc[QLDS ? 1 : RB][QLDS ? 1 : KS_C], qr[QLDS ? 1 : RB][QLDS ? 1 : KS_R];
#pragma unroll
  for (int x = 0; x < RB; ++x) {
    const int rho = (rb * RB + x) * 32 + n;
    row_ok[x] = rho < a.G * a.s_q;
    t_of[x] = row_ok[x] ? rho / a.G : 0;
    head_of[x] = j * a.G + (row_ok[x] ? rho % a.G : 0);
    vis_end[x] = row_ok[x] ? min(ce.tok_end, ce.L - a.s_q + t_of[x] + 1) : 0;  // tokens this row may see in the chunk
    const int64_t qrow = (int64_t)(ce.b * a.s_q + t_of[x]) * a.h_q + head_of[x];
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    const __bf16* pc = (const __bf16*)a.q_a + qrow * DH + h * 8;
    const __bf16* pr = (const __bf16*)a.q_r + qrow * DR + h * 8;
    if constexpr (QLDS) {  // (each lane reads back only what it wrote itself: no barrier needed)
#pragma unroll
      for (int ks = 0; ks < KS_C; ++ks) *(bf16x8*)(q_lds + (x * (KS_C + KS_R) + ks) * 1024) = row_ok[x] ? *(const bf16x8*)(pc + ks * 16) : zero;
#pragma unroll
      for (int ks = 0; ks < KS_R; ++ks) *(bf16x8*)(q_lds + (x * (KS_C + KS_R) + KS_C + ks) * 1024) = row_ok[x] ? *(const bf16x8*)(pr + ks * 16) : zero;
    } else {
#pragma unroll
      for (int ks = 0; ks < KS_C; ++ks) qc[x][ks] = row_ok[x] ? *(const bf16x8*)(pc + ks * 16) : zero;
#pragma unroll
      for (int ks = 0; ks < KS_R; ++ks) qr[x][ks] = row_ok[x] ? *(const bf16x8*)(pr + ks * 16) : zero;
    }
  }
  auto q_content = [&](int x, int ks) __attribute__((always_inline)) -> bf16x8 {
    if constexpr (QLDS) return *(const bf16x8*)(q_lds + (x * (KS_C + KS_R) + ks) * 1024);
    else return qc[x][ks];
  };
  auto q_rope = [&](int x, int ks) __attribute__((always_inline)) -> bf16x8 {
    if constexpr (QLDS) return *(const bf16x8*)(q_lds + (x * (KS_C + KS_R) + KS_C + ks) * 1024);
    else return qr[x][ks];
  };
  const int unmasked_end = min(ce.tok_end, ce.L - a.s_q + 1);             // below this every real row sees every token

  const int P = a.cache.page_size;
  const int gc = a.cache.groups;
  constexpr int EB = FP8 ? 1 : 2;                                             // bytes per K_C / V element
  const int64_t page_bytes = (int64_t)P * (gc * (DH + DV) * EB + DR * 2);
  const int64_t kr_plane = (int64_t)gc * (DH + DV) * P * EB;                   // byte offset of the k_R plane in a page
  const char* pool = (const char*)a.cache.pool;

  bf16x8 kf[KS_C], rf[KS_R], vf[MT][2];
  u32x4 kf8[FP8 ? KS_C / 2 : 1], vf8[FP8 ? MT : 1];                           // raw code vectors (FP8 only)

  bool k_ok = true, v_ok = true;

  // The shared RoPE key of a tile is the same for every group.  When all waves of a workgroup are groups of one
  // (chunk, row block) -- 8 waves for g a multiple of 8, g waves for g = 2 or 4 -- the tile's k_R (4 KB) is brought
  // into LDS once per workgroup, as four 1 KB LDS-DMA instructions dealt over the waves, and every wave takes its
  // fragments from there, instead of every wave pulling the same lines through the vector memory path (a fifth of
  // all its load instructions).
  __shared__ __attribute__((aligned(16))) char kr_lds[2][KS_R * 1024];
  const bool share_kr = share_kr_arg != 0;                                  // kernel-uniform
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);        // position in the workgroup (scalar)
  auto stage_kr = [&](int tok, int32_t pg, int buf) {
    for (int ks = wave; ks < KS_R; ks += wpb) {  // k-step ks: dims 16*ks .. 16*ks + 15
      const char* src = pool + (int64_t)(pg >= 0 ? pg : 0) * page_bytes + kr_plane + ((int64_t)(2 * ks) * P + tok % P) * 16;
      const uint32_t dst = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr_t)(kr_lds[buf] + ks * 1024));
      // ("memory": the cache loads that follow must stay behind this request, the counted wait relies on it)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(dst), "v"((h * P + n) * 16), "s"(src) : "memory");
    }
  };
  auto load_k = [&](int tok, int32_t pg) {
    k_ok = pg >= 0;
    const char* base = pool + (int64_t)(k_ok ? pg : 0) * page_bytes;
    const int slot = tok % P + n;
    const char* kb = base + (int64_t)j * DH * P * EB + ((int64_t)h * P + slot) * 16;   // vector index h (+ 2 per step below)
    const char* rbp = base + kr_plane + ((int64_t)h * P + slot) * 16;
    if constexpr (FP8) {
#pragma unroll
      for (int kp = 0; kp < KS_C / 2; ++kp) kf8[kp] = __builtin_nontemporal_load((const u32x4*)(kb + (int64_t)kp * 32 * P));
    } else {
#pragma unroll
      for (int ks = 0; ks < KS_C; ++ks) kf[ks] = __builtin_nontemporal_load((const bf16x8*)(kb + (int64_t)ks * 32 * P));
    }
    if (!share_kr) {
#pragma unroll
      for (int ks = 0; ks < KS_R; ++ks) rf[ks] = __builtin_nontemporal_load((const bf16x8*)(rbp + (int64_t)ks * 32 * P));
    }
  };
  auto load_v = [&](int tok, int32_t pg) {
    v_ok = pg >= 0;
    const char* base = pool + (int64_t)(v_ok ? pg : 0) * page_bytes + ((int64_t)gc * DH * P + (int64_t)j * DV * P) * EB;
    if constexpr (FP8) {
      const int T = (tok % P) / 32;  // 32-token tile of the page: [T][dim][half] vectors
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        vf8[mt] = __builtin_nontemporal_load((const u32x4*)(base + ((((int64_t)T * DH + mt * 32 + n) * 2 + h) * 16)));
    } else {
      const int tb = (tok % P) / 8 + h;  // 8-token block of this lane for k-step 0; k-step 1 is two blocks further
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
          vf[mt][kk] = __builtin_nontemporal_load((const bf16x8*)(base + ((int64_t)(tb + 2 * kk) * DV + mt * 32 + n) * 16));
    }
  };

  f32x16 o[RB][MT];
  float m_run[RB], l_run[RB];
#pragma unroll
  for (int x = 0; x < RB; ++x) {
    m_run[x] = GQLA_NEG_INF;
    l_run[x] = 0.f;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[x][mt][i] = 0.f;
  }

  // Page ids travel through the scalar cache, looked up one tile ahead of the loads that need them: a vector load of
  // the table entry would have to be waited for with vmcnt(0), i.e. behind every cache load still in flight.
  const int32_t* table_row = a.cache.page_table ? a.cache.page_table + (int64_t)ce.b * a.cache.max_pages : nullptr;
  auto checked = [&](int32_t pg) -> int32_t { return ((uint32_t)pg < (uint32_t)a.cache.num_pages) ? pg : -1; };
  auto lookup_start = [&](int tok, int32_t& raw) {  // asynchronous; lookup_done() must precede any use of raw
    if (table_row) asm volatile("s_load_dword %0, %1, 0x0" : "=s"(raw) : "s"(table_row + tok / P));
    else raw = ce.b * a.cache.max_pages + tok / P;
  };
  auto lookup_done = [&](int32_t& raw) {
    if (table_row) asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(raw));
  };
  int32_t pg_raw = 0;
  int32_t pg_next = -1;
  const int tok0 = ce.tok_begin + 32 * tw;  // this wave's first tile (a short chunk may leave some of a team without any)
  if (tok0 < ce.tok_end) {
    lookup_start(tok0, pg_raw);
    lookup_done(pg_raw);
    pg_next = checked(pg_raw);
    if (share_kr) stage_kr(tok0, pg_next, 0);
    load_k(tok0, pg_next);
    load_v(tok0, pg_next);
    if (tok0 + tstep < ce.tok_end) lookup_start(tok0 + tstep, pg_raw);
  }
  for (int tok = tok0; tok < ce.tok_end; tok += tstep) {
    f32x16 s[RB];
#pragma unroll
    for (int x = 0; x < RB; ++x)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[x][i] = 0.f;
    if constexpr (FP8) {
#pragma unroll
      for (int kp = 0; kp < KS_C / 2; ++kp) {
        kf[2 * kp] = widen_e4m3(kf8[kp][0], kf8[kp][1]);
        kf[2 * kp + 1] = widen_e4m3(kf8[kp][2], kf8[kp][3]);
      }
      // the value codes are widened here as well: their registers are then free for the next tile's codes, which are
      // requested together with the key codes (twice the bytes in flight per wave)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        vf[mt][0] = widen_e4m3(vf8[mt][0], vf8[mt][1]);
        vf[mt][1] = widen_e4m3(vf8[mt][2], vf8[mt][3]);
      }
    }
    const bool tile_v_ok = v_ok;  // v_ok is overwritten by the next tile's request below (FP8)

#pragma unroll
    for (int ks = 0; ks < KS_C; ++ks)
#pragma unroll
      for (int x = 0; x < RB; ++x) s[x] = mfma32(kf[ks], q_content(x, ks), s[x]);
    if constexpr (FP8) {
#pragma unroll
      for (int x = 0; x < RB; ++x)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[x][i] *= k_scale;
    }
    if (share_kr) {
      // this tile's k_R was requested before the cache loads that followed it (loads complete in issue order): the
      // tile's key and value vectors, 16-byte loads each -- KS_C + 2*MT of them in 16 bits, half as many as codes
      constexpr int kLoadsBehindKr = FP8 ? KS_C / 2 + MT : KS_C + 2 * MT;
      static_assert(kLoadsBehindKr == 8 || kLoadsBehindKr == 16 || kLoadsBehindKr == 28, "the wait below is written for these counts");
      if constexpr (kLoadsBehindKr == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
      else if constexpr (kLoadsBehindKr == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(28)" ::: "memory");
      __syncthreads();
      const char* kr = kr_lds[((tok - ce.tok_begin) >> 5) & 1] + lane * 16;
#pragma unroll
      for (int ks = 0; ks < KS_R; ++ks) rf[ks] = *(const bf16x8*)(kr + ks * 1024);
    }
#pragma unroll
    for (int ks = 0; ks < KS_R; ++ks)
#pragma unroll
      for (int x = 0; x < RB; ++x) s[x] = mfma32(rf[ks], q_rope(x, ks), s[x]);
    const bool tile_k_ok = k_ok;
    const bool has_next = tok + tstep < ce.tok_end;
    if (has_next) {
      lookup_done(pg_raw);
      pg_next = checked(pg_raw);
      if (share_kr) stage_kr(tok + tstep, pg_next, (((tok - ce.tok_begin) >> 5) + 1) & 1);  // (shared k_R: tt = 1)
      load_k(tok + tstep, pg_next);
      if constexpr (FP8) load_v(tok + tstep, pg_next);
      if (tok + 2 * tstep < ce.tok_end) lookup_start(tok + 2 * tstep, pg_raw);
    }

    // online softmax, base-2 domain; register i of lane (n, h) is token tok + 8*(i/4) + 4*h + i%4
    bf16x8 pf[RB][2];
#pragma unroll
    for (int x = 0; x < RB; ++x) {
      float sv[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) sv[i] = s[x][i] * a.scale_log2e;
      const bool need_mask = (tok + 32 > unmasked_end) || !tile_k_ok || !row_ok[x];
      if (need_mask) {
        const int lim = tile_k_ok ? vis_end[x] : 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int tk = tok + 8 * (i >> 2) + 4 * h + (i & 3);
          if (tk >= lim) sv[i] = GQLA_NEG_INF;
        }
      }
      float tmax = sv[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, sv[i]);
      tmax = pair_max(tmax);
      // m_run is the reference of the exponentials, not the exact running maximum: it moves only when some row's
      // maximum has outgrown it by kRescaleThreshold (log2 units; the probabilities then stay below 2^threshold, far
      // inside the range of bf16 and fp32), so that far into a long context the update of O^T and l is skipped
      if (__builtin_amdgcn_ballot_w64(tmax > m_run[x] + kRescaleThreshold) != 0) {
        const float m_new = fmaxf(m_run[x], tmax);
        const float alpha = fast_exp2(m_run[x] - ((m_new == GQLA_NEG_INF) ? 0.f : m_new));
        m_run[x] = m_new;
        l_run[x] *= alpha;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[x][mt][i] *= alpha;
      }
      const float m_use = (m_run[x] == GQLA_NEG_INF) ? 0.f : m_run[x];
#pragma unroll
      for (int i = 0; i < 16; ++i) sv[i] = fast_exp2(sv[i] - m_use);

      // P^T fragments: k-step kk covers tokens tok + 16*kk .. +15, lane half h needs tokens 8h .. 8h+7 of them.
      // The denominator sums the probabilities as the matrix cores see them (rounded to bf16): numerator and
      // denominator then weigh every token alike, whatever the reference of the exponentials is.
      float psum = 0.f;
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const uint32_t x0 = pack_bf16(sv[8 * kk + 0], sv[8 * kk + 1]), x1 = pack_bf16(sv[8 * kk + 2], sv[8 * kk + 3]);
        const uint32_t y0 = pack_bf16(sv[8 * kk + 4], sv[8 * kk + 5]), y1 = pack_bf16(sv[8 * kk + 6], sv[8 * kk + 7]);
#pragma unroll
        for (uint32_t wd : {x0, x1, y0, y1}) psum += __builtin_bit_cast(float, wd << 16) + __builtin_bit_cast(float, wd & 0xffff0000u);
        u32x4 w;
        uint32_t r0, r1;
        half_swap(x0, y0, r0, r1);
        w[0] = r0;
        w[2] = r1;
        half_swap(x1, y1, r0, r1);
        w[1] = r0;
        w[3] = r1;
        pf[x][kk] = __builtin_bit_cast(bf16x8, w);
      }
      l_run[x] += psum;  // per-lane partial sum; the two half-waves are added at the end
    }

    // values of tokens outside the chunk may hold any bits (NaN included): zero them so that 0 * v stays 0
    if (tok + 32 > ce.tok_end || !tile_v_ok) {
      const int lim = tile_v_ok ? ce.tok_end : 0;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (tok + 16 * kk + 8 * h + e >= lim) vf[mt][kk][e] = (__bf16)0.f;
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int x = 0; x < RB; ++x) o[x][mt] = mfma32(vf[mt][kk], pf[x][kk], o[x][mt]);
    if constexpr (!FP8) {
      if (has_next) load_v(tok + tstep, pg_next);
    }
  }

  if constexpr (CAN_TEAM) {
    if (tt > 1) {
      // ---- merge of the team's partial states (tt = 8 waves; row = lane % 32) ----
      // dyn_lds: O^T of every wave as [wave][quad q = 4 mt + i/4][lane][4] fp32 (16 KB per wave, MT = 4), then m and l
      // per (wave, row).  Wave w sums quads 2w, 2w + 1 of all eight waves in a fixed order and writes them.
      constexpr int kQuads = MT * 4;
      float* const o_lds = (float*)dyn_lds;
      float* const ml_lds = o_lds + 8 * kQuads * 64 * 4;
      const float l_mine = pair_sum(l_run[0]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          *(f32x4*)(o_lds + ((tw * kQuads + 4 * mt + q) * 64 + lane) * 4) =
              f32x4{o[0][mt][4 * q], o[0][mt][4 * q + 1], o[0][mt][4 * q + 2], o[0][mt][4 * q + 3]};
      if (h == 0) {
        ml_lds[tw * 32 + n] = m_run[0];
        ml_lds[256 + tw * 32 + n] = l_mine;
      }
      __syncthreads();
      float m_all = GQLA_NEG_INF;
#pragma unroll
      for (int w = 0; w < 8; ++w) m_all = fmaxf(m_all, ml_lds[w * 32 + n]);
      const float m_use = (m_all == GQLA_NEG_INF) ? 0.f : m_all;
      float c[8], l_all = 0.f;
#pragma unroll
      for (int w = 0; w < 8; ++w) {
        c[w] = fast_exp2(ml_lds[w * 32 + n] - m_use);  // 0 for a wave that saw no visible token
        l_all += c[w] * ml_lds[256 + w * 32 + n];
      }
      const bool ok = row_ok[0];
      const float inv = (l_all > 0.f ? 1.f / l_all : 0.f) * (FP8 ? v_scale : 1.f);
      const int rho = t_of[0] * a.h_q + head_of[0];
      const int64_t prow = (int64_t)chunk * a.M + rho;
      // chunk partial in fp32, 4-dim vectors ordered [chunk][32-row block][d_v / 4][row] (part_vec_index): this lane
      // holds vector 2 quad + h of its row
      float* po = (float*)a.part_o + part_vec_index(chunk, rho, a.M, DV / 4, h) * 4;
      constexpr int kQuadsPerWave = kQuads / 8;
      static_assert(kQuads % 8 == 0, "every wave of the team sums the same number of quads");
#pragma unroll
      for (int qq = 0; qq < kQuadsPerWave; ++qq) {
        const int quad = tw * kQuadsPerWave + qq;  // = 4 mt + q
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < 8; ++w) {
          const f32x4 v = *(const f32x4*)(o_lds + ((w * kQuads + quad) * 64 + lane) * 4);
          if (c[w] > 0.f) acc += c[w] * v;  // (a wave without tiles holds zeros; one whose rows were all masked may hold anything times 0)
        }
        acc *= inv;
        if (ok) *(f32x4*)(po + 2 * quad * (32 * 4)) = acc;
      }
      if (ok && tw == 0 && h == 0) a.part_lse[prow] = l_all > 0.f ? (m_all + fast_log2(l_all)) * kLn2 : GQLA_NEG_INF;
      return;
    }
  }

#pragma unroll
  for (int x = 0; x < RB; ++x) {
    const float l_tot = pair_sum(l_run[x]);
    if (!row_ok[x]) continue;
    const float inv = (l_tot > 0.f ? 1.f / l_tot : 0.f) * (FP8 ? v_scale : 1.f);
    const int rho = t_of[x] * a.h_q + head_of[x];
    const int64_t prow = (int64_t)chunk * a.M + rho;
    // chunk partial in fp32, 4-dim vectors ordered [chunk][32-row block][d_v / 4][row] (part_vec_index): consecutive rows
    // sit in consecutive lanes, so a store instruction writes runs of contiguous 16-byte vectors instead of 32-byte pieces
    // of 32 rows; all waves of the launch reach this point together, and nothing hides what these stores cost.  (16-bit
    // partials would halve them, but cost the path its margin on outputs of magnitude 4 to 8, where half a bf16 step
    // of the final rounding alone is 1.6e-2 of the 2e-2 allowed.)
    float* po = (float*)a.part_o + part_vec_index(chunk, rho, a.M, DV / 4, h) * 4;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *(f32x4*)(po + (8 * mt + 2 * q) * (32 * 4)) =
            f32x4{o[x][mt][4 * q] * inv, o[x][mt][4 * q + 1] * inv, o[x][mt][4 * q + 2] * inv, o[x][mt][4 * q + 3] * inv};
    if (h == 0) a.part_lse[prow] = l_tot > 0.f ? (m_run[x] + fast_log2(l_tot)) * kLn2 : GQLA_NEG_INF;
  }
}


// ---- log-sum-exp merge of the chunk partials (not in the paper: the split over the context is this library's) ----------
// One workgroup per (sequence, block of 32 rows); thread (row n = tid % 32, vector slot tid / 32) merges vectors
// slot, slot + 8, ... of its row (4 floats each), so that the loads of a wave are 32 consecutive 16-byte vectors.
// Chunks are merged kNB at a time (their loads in flight together) with a running maximum, as in an online softmax.  The
// merged block goes through LDS (32 rows, padded) and leaves as whole rows: 16 lanes x 16 bytes per row of 128 value dims.
template <int DV>
__global__ void __launch_bounds__(256) combine_gqa_bf16_kernel(CombineArgs a) {
  constexpr int kNB = 4;
  constexpr int NV = DV / 4;                 // 4-float vectors per row
  constexpr int PITCH = DV * 2 + 16;         // bytes per row of the block in LDS
  __shared__ __attribute__((aligned(16))) char tile[32 * PITCH];
  const int blocks_per_seq = (a.M + 31) / 32;
  const int b = blockIdx.x / blocks_per_seq, rb = blockIdx.x % blocks_per_seq;
  const int n = threadIdx.x & 31, slot = threadIdx.x >> 5;
  const int rho = rb * 32 + n;
  const bool row_ok = rho < a.M;
  const int rc = row_ok ? rho : 0;
  const int s0 = a.first_slot[b], s1 = a.first_slot[b + 1];
  const f32x4* po = (const f32x4*)a.part_o + part_vec_index(0, rc, a.M, NV, slot);
  const int64_t chunk_stride = (int64_t)blocks_per_seq * NV * 32;   // vectors from one chunk's partials to the next
  float m = GQLA_NEG_INF, den = 0.f;
  f32x4 acc[NV / 8];
#pragma unroll
  for (int v = 0; v < NV / 8; ++v) acc[v] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int sb = s0; sb < s1; sb += kNB) {
    float l[kNB];
    f32x4 x[kNB][NV / 8];
#pragma unroll
    for (int k = 0; k < kNB; ++k) {
      const int sc = min(sb + k, s1 - 1);  // clamped: a chunk beyond the range is loaded again and given weight 0
      l[k] = a.part_lse[(int64_t)sc * a.M + rc];
#pragma unroll
      for (int v = 0; v < NV / 8; ++v) x[k][v] = po[sc * chunk_stride + v * (8 * 32)];
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
#pragma unroll
    for (int v = 0; v < NV / 8; ++v) acc[v] *= rescale;
    m = m_new;
#pragma unroll
    for (int k = 0; k < kNB; ++k) {
      const float w = __expf(l[k] - m_use);
      den += w;
      if (w > 0.f) {  // a chunk without visible tokens may hold anything
#pragma unroll
        for (int v = 0; v < NV / 8; ++v) acc[v] += w * x[k][v];
      }
    }
  }
  const float inv = den > 0.f ? 1.f / den : 0.f;
#pragma unroll
  for (int v = 0; v < NV / 8; ++v)
    *(u32x2*)(tile + n * PITCH + (slot + 8 * v) * 8) = u32x2{pack_bf16(acc[v][0] * inv, acc[v][1] * inv), pack_bf16(acc[v][2] * inv, acc[v][3] * inv)};
  if (a.lse && row_ok && slot == 0) a.lse[(int64_t)b * a.M + rho] = m + __logf(den);
  __syncthreads();
  constexpr int LPR = DV / 8;                // lanes per row on the way out (16 bytes each)
  for (int idx = threadIdx.x; idx < 32 * LPR; idx += 256) {
    const int r = idx / LPR, c = idx % LPR;
    if (rb * 32 + r < a.M)
      *(u32x4*)((__bf16*)a.out + ((int64_t)b * a.M + rb * 32 + r) * DV + c * 8) = *(const u32x4*)(tile + r * PITCH + c * 16);
  }
}

}  // namespace

// rows_per_wave: 32, or 64 when a wave takes two row blocks
static void gqa_launch_shape(const DecodeArgs& a, int max_wpb, int rows_per_wave, int& row_blocks, int& n_items, bool& team, int& wpb,
                             int& blocks) {
  row_blocks = (a.G * a.s_q + rows_per_wave - 1) / rows_per_wave;
  n_items = a.n_chunks * row_blocks * a.g;
  // all waves of a workgroup are groups of one (chunk, row block) when the group count is a multiple of the waves per
  // workgroup: then they share the tile's k_R through LDS (and run in step, one barrier per tile)
  // With 2 or 4 groups the workgroup also takes all row blocks of the chunk when that keeps it within its waves: they
  // stream the same cache vectors in step, so all but the first request for a line is served by the cache hierarchy.
  const bool few = (a.g == 4 || a.g == 2) && a.g <= max_wpb;
  team = a.g % max_wpb == 0 || few;
  wpb = few ? (a.g * row_blocks <= max_wpb ? a.g * row_blocks : a.g) : max_wpb;
  blocks = (n_items + wpb - 1) / wpb;
}

template <bool FP8>
static hipError_t launch_decode_gqa_128(const DecodeArgs& a, float k_scale, float v_scale, hipStream_t s) {
  int row_blocks, n_items, wpb, blocks;
  bool team;
  if (a.G * a.s_q > 32) {  // more than one row block per group: two per wave, four waves per workgroup
    gqa_launch_shape(a, 4, 64, row_blocks, n_items, team, wpb, blocks);
    constexpr int kQBytesPerWave = 2 * (128 / 16 + 64 / 16) * 1024;  // both row blocks' query fragments
    static const hipError_t attr = hipFuncSetAttribute((const void*)decode_gqa_bf16_kernel<128, 128, 64, FP8, 256, 2>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, 4 * kQBytesPerWave);
    if (attr != hipSuccess) return attr;
    decode_gqa_bf16_kernel<128, 128, 64, FP8, 256, 2><<<blocks, 64 * wpb, wpb * kQBytesPerWave, s>>>(a, n_items, row_blocks, team ? 1 : 0,
                                                                                                    1, k_scale, v_scale);
    return hipGetLastError();
  }
  if (a.g == 1) {  // one group with at most 32 query rows: a token team of eight waves per chunk (the plan cuts chunks for that)
    constexpr int kMergeBytes = 8 * (128 / 32) * 4 * 64 * 16 + 2 * 8 * 32 * 4;  // eight O^T of 16 KB, then m and l per (wave, row)
    static const hipError_t attr = hipFuncSetAttribute((const void*)decode_gqa_bf16_kernel<128, 128, 64, FP8, 512, 1>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kMergeBytes);
    if (attr != hipSuccess) return attr;
    decode_gqa_bf16_kernel<128, 128, 64, FP8, 512, 1><<<a.n_chunks, 512, kMergeBytes, s>>>(a, a.n_chunks, 1, 0, 8, k_scale, v_scale);
    return hipGetLastError();
  }
  gqa_launch_shape(a, 8, 32, row_blocks, n_items, team, wpb, blocks);
  decode_gqa_bf16_kernel<128, 128, 64, FP8, 512, 1><<<blocks, 64 * wpb, 0, s>>>(a, n_items, row_blocks, team ? 1 : 0, 1, k_scale, v_scale);
  return hipGetLastError();
}

hipError_t launch_decode_gqa_bf16(const DecodeArgs& a, hipStream_t s) {
  if (a.d_h == 192) {  // (d_h, d_v) = (192, 256): four waves per workgroup, one row block each
    int row_blocks, n_items, wpb, blocks;
    bool team;
    gqa_launch_shape(a, 4, 32, row_blocks, n_items, team, wpb, blocks);
    decode_gqa_bf16_kernel<192, 256, 64, false, 256, 1><<<blocks, 64 * wpb, 0, s>>>(a, n_items, row_blocks, team ? 1 : 0, 1, 1.f, 1.f);
    return hipGetLastError();
  }
  return launch_decode_gqa_128<false>(a, 1.f, 1.f, s);
}

hipError_t launch_decode_gqa_fp8(const DecodeArgs& a, float k_scale, float v_scale, hipStream_t s) {
  return launch_decode_gqa_128<true>(a, k_scale, v_scale, s);
}

hipError_t launch_combine_gqa_bf16(const CombineArgs& a, hipStream_t s) {
  const unsigned blocks = (unsigned)(a.B * ((a.M + 31) / 32));
  if (a.d_h == 256) combine_gqa_bf16_kernel<256><<<blocks, 256, 0, s>>>(a);   // a.d_h: value dims here
  else combine_gqa_bf16_kernel<128><<<blocks, 256, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace gqla
