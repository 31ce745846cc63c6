// MQA-absorb split-L decode over the latent cache, bf16 MFMA (paper Sec. 3.1, MQA-absorb equation, lines 2-5).
//
// One workgroup of 4 waves per (chunk, block of 128 query rows); wave w owns rows 32w..32w+31 of the block.
// A 32-token latent tile [32][r_kv + d_r] is staged once into LDS (global_load_lds into a ring of four tile
// buffers, three tiles ahead of its use) and serves every row of the block twice: row-wise as the key operand
// [c | k_R] and transposed (ds_read_b64_tr_b16) as the value operand c:
//   S^T[token][row]  = Kt[token][576] * Qhat^T[576][row]      A = LDS row fragments,   B = queries in registers
//   O^T[r][row]     += C^T[r][token]  * P^T[token][row]       A = LDS transposed frags, B = probabilities
// O^T (512 x 32 fp32 per wave) lives in the 256 accumulation registers, addressed by name (see acc_* below); the
// softmax reference maximum is only moved (and O^T rescaled) when a row's maximum grows by more than 2^8, so that
// rescaling is rare.
// Each chunk's normalised latent-space output is written as bf16 with its log-sum-exp; the combine kernel merges
// chunks and applies W_UV.  Intensity h_q s_q (2 r_kv + d_r) / (r_kv + d_r) (Sec. 4.2.1): 242 FLOP/byte for 128 rows,
// 484 for 256 (s_q = 2), against a ridge of about 310 on this chip.
#include "gqla_device.h"
#include "gqla_lds.h"

namespace gqla {

namespace {

constexpr int kTile = 32;                 // tokens per LDS tile
constexpr int kSlots = 4;                 // tile buffers in the LDS ring
constexpr int kRowsPerBlock = 128;        // query rows per workgroup
constexpr float kRescaleThreshold = 8.f;  // log2 units

// ---- O^T accumulators, managed by hand ----
// O^T (512 x 32 fp32 per wave) fills all 256 accumulation registers: tile dt (32 latent dims x 32 rows) is a[16*dt : 16*dt+15].
// They are addressed by NAME in inline assembly and never appear as C++ values: the compiler then has nothing to
// allocate, copy or spill there, and the rest of the kernel gets the 256 ordinary registers to itself.  Every statement
// below is `asm volatile`, so they keep their program order; the callers keep the hardware's timing rules
// (results of an MFMA are read by non-MFMA instructions only after its last pass has long retired).
#define GQLA_ACC(D) "a[" #D "*16:" #D "*16+15]"
#define GQLA_FOR_DT(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15)

__device__ __forceinline__ void acc_zero() {
  asm volatile(".set gqla_i, 0\n.rept 256\n\tv_accvgpr_write_b32 a[gqla_i], 0\n.set gqla_i, gqla_i+1\n.endr" : : : GQLA_ALL_AGPRS);
}
// O^T tile dt += A * B (dt is a compile-time value at every call site: the switch folds away)
__device__ __forceinline__ void acc_mfma(int dt, bf16x8 a, bf16x8 b) {
  switch (dt) {
#define X(D) case D: asm volatile("v_mfma_f32_32x32x16_bf16 " GQLA_ACC(D) ", %0, %1, " GQLA_ACC(D) : : "v"(a), "v"(b)); break;
    GQLA_FOR_DT(X)
#undef X
  }
}
// every accumulator of this lane times alpha (one query row per lane, so alpha is per lane)
__device__ __forceinline__ void acc_scale(float alpha) {
  float t0, t1;
  asm volatile(
      ".set gqla_i, 0\n.rept 128\n"
      "\tv_accvgpr_read_b32 %0, a[gqla_i]\n\tv_accvgpr_read_b32 %1, a[gqla_i+1]\n"
      "\tv_mul_f32 %0, %0, %2\n\tv_mul_f32 %1, %1, %2\n\ts_nop 0\n"
      "\tv_accvgpr_write_b32 a[gqla_i], %0\n\tv_accvgpr_write_b32 a[gqla_i+1], %1\n"
      ".set gqla_i, gqla_i+2\n.endr"
      : "=&v"(t0), "=&v"(t1)
      : "v"(alpha));
}
// tile dt into 16 ordinary registers (first call after the last MFMA: pass wait = true)
__device__ __forceinline__ void acc_read(int dt, bool wait, float (&x)[16]) {
  if (wait) asm volatile("s_nop 15\n\ts_nop 7");
  switch (dt) {
#define X(D)                                                                                                            \
  case D:                                                                                                               \
    asm volatile(".set gqla_i, 0\n.irp r, %0, %1, %2, %3, %4, %5, %6, %7, %8, %9, %10, %11, %12, %13, %14, %15\n"        \
                 "\tv_accvgpr_read_b32 \\r, a[" #D "*16+gqla_i]\n.set gqla_i, gqla_i+1\n.endr"                           \
                 : "=v"(x[0]), "=v"(x[1]), "=v"(x[2]), "=v"(x[3]), "=v"(x[4]), "=v"(x[5]), "=v"(x[6]), "=v"(x[7]),      \
                   "=v"(x[8]), "=v"(x[9]), "=v"(x[10]), "=v"(x[11]), "=v"(x[12]), "=v"(x[13]), "=v"(x[14]), "=v"(x[15])); \
    break;
    GQLA_FOR_DT(X)
#undef X
  }
}

// SPLIT = 1: the layout above.  SPLIT = 4 (at most 32 query rows per sequence, e.g. one rank's heads under tensor
// parallelism; or so few chunks that one workgroup per 32 rows still fits the chip in one round): the four waves
// share a block of 32 rows instead of owning 32 rows each.  A wave of
// the team contracts a quarter of the key dimension (k-step `part` of each 4-step panel), the team sums its partial
// S^T through LDS (every wave adds them in the same order, so all hold the same bits), each wave runs the same
// softmax and then updates its own RKV/4 slice of O^T.  With so few rows the kernel is bound by the rate at which
// tiles stream into LDS (measured: 64 rows gain nothing from two-wave teams, so those keep SPLIT = 1).
template <int RKV, int DR, int SPLIT>
__global__ void __launch_bounds__(256) decode_absorb_bf16_kernel(DecodeArgs a, int row_blocks) {
  constexpr int W = RKV + DR;        // elements per latent row
  constexpr int ROWB = W * 2;        // bytes per latent row
  constexpr int NP = W / 64;         // 128-byte panels per latent row
  constexpr int PANEL = kTile * 128; // bytes per panel
  constexpr int KS = W / 16;         // k-steps of the key contraction
  constexpr int DT = RKV / 32;       // 32-wide tiles of the latent output
  constexpr int TILE_BYTES = kTile * ROWB;
  constexpr int RPB = kRowsPerBlock / SPLIT;  // query rows per workgroup
  constexpr int KB = 4 / SPLIT;               // k-steps of every 4-step panel that one wave contracts
  constexpr int DTW = DT / SPLIT;             // output tiles per wave
  static_assert(SPLIT == 1 || SPLIT == 4, "one wave or the whole workgroup per 32 rows");
  static_assert(W % 64 == 0 && RKV % 64 == 0, "latent row must be a whole number of 128-byte panels");
  static_assert((16 + 8 + 4) * 128 + 128 + PANEL * (RKV / 64 - 1) < 65536, "value-fragment offsets must fit the 16-bit LDS immediate");
  extern __shared__ __attribute__((aligned(16))) char smem[];

  // blockIdx -> (chunk, row block): the row blocks of one chunk get ids that are equal modulo 8 so that they run on
  // the same XCD (ids are dealt round-robin over the 8 XCDs) and share the chunk's cache lines in that XCD's L2.
  int chunk, rbk;
  {
    const int id = blockIdx.x;
    const int grp = id / (8 * row_blocks), rem = id % (8 * row_blocks);
    rbk = rem / 8;
    chunk = grp * 8 + rem % 8;
  }
  if (chunk >= a.n_chunks) return;  // whole workgroup leaves together
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform by construction: keep it scalar
  const int n = lane & 31, h = lane >> 5;
  const ChunkEntry ce = a.chunks[chunk];

  const int part = wave & (SPLIT - 1), team = wave / SPLIT;  // this wave's share of its 32 rows' work; which 32 rows
  const int rho = rbk * RPB + team * 32 + n;                 // row = t * h_q + i
  const bool row_ok = rho < a.M;
  const int t = row_ok ? rho / a.h_q : 0;
  const int vis_end = row_ok ? min(ce.tok_end, ce.L - a.s_q + t + 1) : 0;
  const int unmasked_end = min(ce.tok_end, ce.L - a.s_q + 1);
  // With SPLIT > 1 a workgroup is one team, and the launcher only makes row blocks that have rows (all waves meet
  // at the team's exchange barrier, so none may skip a tile).
  const bool wave_active = SPLIT > 1 || rbk * RPB + team * 32 < a.M;

  const int P = a.cache.page_size;
  const char* pool = (const char*)a.cache.pool;
  // Tiles are always staged whole: rows past the chunk end still come from the page (allocated memory), an
  // out-of-pool page id falls back to page 0; such rows are zeroed in LDS before use (see the loop).
  const int32_t* table_row = a.cache.page_table ? a.cache.page_table + (int64_t)ce.b * a.cache.max_pages : nullptr;
  auto checked = [&](int32_t pg) -> int32_t { return ((uint32_t)pg < (uint32_t)a.cache.num_pages) ? pg : -1; };
  auto tile_src = [&](int32_t pg, int slot) -> const char* {  // first row of a tile: page pg (or page 0), slot `slot`
    return pool + ((int64_t)(pg >= 0 ? pg : 0) * P + slot) * ROWB;
  };

  // Per-lane LDS byte offsets inside a tile (panel layout of gqla_lds.h; everything else is a compile-time offset):
  //  key fragments     row n, chunk 2*ks + h with ks = 4*a4 + b: panel a4, in-panel chunk 2*b + h
  //                    -> four bases (b = 0..3), plus a4*PANEL.
  //  value fragments   (transposed reads) this lane addresses row R0 + 4*h + e (and 8 rows further for the second read),
  //                    4 columns at 32*dt + 16*g1 + 4*q: panel dt/2, in-panel chunk 4*(dt & 1) + cl, cl = 2*g1 + q/2.
  //                    With R0 a multiple of 16, swz = 2*h + e/2 for the first read and 4 + that for the second, so the
  //                    chunk lands at 4*(dt & 1) + (cl ^ swz) resp. 4*(1 - (dt & 1)) + (cl ^ swz): one base per lane.
  uint32_t kbase[KB], vbase;
  {
#pragma unroll
    for (int b = 0; b < KB; ++b) kbase[b] = n * 128 + (((2 * (part * KB + b) + h) ^ lds_swz(n)) << 4);
    const int i16 = lane & 15, e = i16 >> 2, q = i16 & 3, g1 = (lane >> 4) & 1;
    vbase = (4 * h + e) * 128 + (((2 * g1 + (q >> 1)) ^ (2 * h + (e >> 1))) << 4) + (q & 1) * 8;
    vbase += part * (DTW / 2) * PANEL;  // this wave's output tiles are part*DTW .. part*DTW + DTW-1
  }

  static_assert(DT == 16, "O^T fills the 256 accumulation registers exactly");
  acc_zero();
  float m_ref = GQLA_NEG_INF, l_run = 0.f;

  // Ring of kSlots tile buffers.  Tile it + kAhead is staged (9 LDS-DMA instructions per wave, after the S phase)
  // while tile `it` is worked on, so every load has about three tile times to land and only a few KB per wave are
  // ever requested at once.  Loads complete in issue order, so "tile `it` has landed" is a count:
  // at most the instructions of the tiles staged after it may still be outstanding.  No other vector-memory
  // instruction is issued inside the loop: page ids come through the scalar cache, one tile ahead of their use.
  constexpr int kAhead = kSlots - 1;
  constexpr int kStageSteps = NP * (kTile / 8 / 4);  // LDS-DMA instructions per wave and tile
  static_assert(kStageSteps == 9, "the wait counts below assume 9 instructions per wave and tile");
  const int n_tiles = (ce.tok_end - ce.tok_begin + kTile - 1) / kTile;
  // page ids of tiles it, it+1, it+2 (staged) and it+3 (staged during tile it); the four first lookups go out together
  // (indices clamped to the chunk's last page, results of tiles that do not exist discarded)
  int32_t pg0, pg1, pg2, pg3;
  {
    const int p_last = (ce.tok_end - 1) / P;
    int32_t raw[4];
    if (table_row) {  // four scalar loads in flight together, one wait
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int p = __builtin_amdgcn_readfirstlane(min(ce.tok_begin / P + (k * kTile) / P, p_last));
        asm volatile("s_load_dword %0, %1, 0x0" : "=s"(raw[k]) : "s"(table_row + p) : "memory");
      }
      asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(raw[0]), "+s"(raw[1]), "+s"(raw[2]), "+s"(raw[3]) : : "memory");
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) raw[k] = ce.b * a.cache.max_pages + min(ce.tok_begin / P + (k * kTile) / P, p_last);
    }
    pg0 = checked(raw[0]);
    pg1 = n_tiles > 1 ? checked(raw[1]) : -1;
    pg2 = n_tiles > 2 ? checked(raw[2]) : -1;
    pg3 = n_tiles > 3 ? checked(raw[3]) : -1;
  }
  int32_t pg_raw = 0;  // table entry of tile it + 4, in flight through the scalar cache
  // Chunks start on a page boundary and pages hold a whole number of tiles: (page index, slot) of the tiles ahead are
  // advanced by addition, and the table is consulted once per page.
  const int p_first = ce.tok_begin / P;
  int st_slot = (kAhead * kTile) % P;                                       // slot of tile it + 3 in its page
  int lk_slot = ((kAhead + 1) * kTile) % P, lk_p = p_first + ((kAhead + 1) * kTile) / P;  // tile it + 4
  static_assert(kAhead == 3, "the page-id shift register holds four tiles");
  stage_panels_full<kTile, NP, 4, ROWB>(smem, tile_src(pg0, 0), wave, lane);
  if (n_tiles > 1) stage_panels_full<kTile, NP, 4, ROWB>(smem + TILE_BYTES, tile_src(pg1, kTile % P), wave, lane);
  if (n_tiles > 2) stage_panels_full<kTile, NP, 4, ROWB>(smem + 2 * TILE_BYTES, tile_src(pg2, (2 * kTile) % P), wave, lane);

  // queries of this lane's row, as B fragments: [q_hat (RKV) | q_R (DR)], 8 consecutive dims per k-step; this wave's
  // k-steps are 4*a4 + part*KB + b
  bf16x8 qf[KS / SPLIT];
  {
    const int64_t qrow = (int64_t)ce.b * a.M + min(rho, a.M - 1);
    const __bf16* ph = (const __bf16*)a.q_a + qrow * RKV + h * 8 + part * KB * 16;
    const __bf16* pr = (const __bf16*)a.q_r + qrow * DR + h * 8 + part * KB * 16;
#pragma unroll
    for (int a4 = 0; a4 < KS / 4; ++a4)
#pragma unroll
      for (int b = 0; b < KB; ++b)
        qf[a4 * KB + b] = *(const bf16x8*)((a4 < RKV / 64 ? ph + a4 * 64 : pr + (a4 - RKV / 64) * 64) + b * 16);
  }

  // The query loads go out behind the first tile requests (one memory latency for both) and are made to complete
  // here, before the loop.  Otherwise the compiler, which counts only the loads it issued itself, keeps "wait for
  // the query loads" counts in front of the loop's first MFMAs; on the hardware counter those waits would also
  // cover the tile requests in flight and drain the ring on every tile.  (The wait that the compiler places here
  // covers the three tiles requested above as well; the loop's own counted waits then pass at once for them.)
#pragma unroll
  for (int k = 0; k < KS / SPLIT; k += 9)
    asm volatile("" : "+v"(qf[k]), "+v"(qf[k + 1]), "+v"(qf[k + 2]), "+v"(qf[k + 3]), "+v"(qf[k + 4]), "+v"(qf[k + 5]),
                      "+v"(qf[k + 6]), "+v"(qf[k + 7]), "+v"(qf[k + 8]));
  static_assert((KS / SPLIT) % 9 == 0, "query fragments are touched nine at a time");

#pragma unroll 1
  for (int it = 0; it < n_tiles; ++it) {
    const int tok = ce.tok_begin + it * kTile;
    const char* buf = smem + (it & (kSlots - 1)) * TILE_BYTES;
    // everything that does not need the tile goes before the wait for it
    const bool stage_next = it + kAhead < n_tiles;
    const char* next_g = tile_src(stage_next ? pg3 : 0, st_slot);
    char* next_buf = smem + ((it + kAhead) & (kSlots - 1)) * TILE_BYTES;
    const bool lookup = it + kAhead + 1 < n_tiles;
    const bool new_page = lookup && lk_slot == 0;
    if (new_page && table_row)  // scalar load, consumed at the end of the tile (its wait is written out there)
      asm volatile("s_load_dword %0, %1, 0x0" : "=s"(pg_raw) : "s"(table_row + lk_p) : "memory");
    {
      const int behind = min(kAhead - 1, n_tiles - 1 - it);  // tiles staged after this one
      if (behind >= 2) asm volatile("s_waitcnt vmcnt(18)" ::: "memory");
      else if (behind == 1) asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();  // tile `it` has landed for every wave; every wave is done reading tile it-1
    const bool tile_ok = pg0 >= 0;
    const int valid = tile_ok ? min(kTile, ce.tok_end - tok) : 0;
    if (valid < kTile) {
      // rows past the chunk end hold whatever the page holds (NaN bits included): zero them so that 0 * v stays 0
      for (int idx = threadIdx.x; idx < (kTile - valid) * (W / 8); idx += 256) {
        const int r = valid + idx / (W / 8), c = idx % (W / 8);
        *(u32x4*)(smem + (it & (kSlots - 1)) * TILE_BYTES + (c >> 3) * PANEL + r * 128 + (c & 7) * 16) = u32x4{0u, 0u, 0u, 0u};
      }
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
      __syncthreads();
    }

    auto shift_pages = [&]() {  // tile it+1 becomes current; the page of tile it + 4 joins the window
      if (new_page && table_row) asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(pg_raw) : : "memory");
      pg0 = pg1;
      pg1 = pg2;
      pg2 = pg3;
      if (new_page) pg3 = checked(table_row ? pg_raw : ce.b * a.cache.max_pages + lk_p);
      if (!lookup) pg3 = -1;
      st_slot = lk_slot;
      lk_slot += kTile;
      if (lk_slot == P) {
        lk_slot = 0;
        ++lk_p;
      }
    };
    if (!wave_active) {  // waves without query rows only help staging (uniform per wave): their share, in one burst
      if (stage_next) stage_panels_full<kTile, NP, 4, ROWB>(next_buf, next_g, wave, lane);
      shift_pages();
      continue;
    }
    {
      const bool need_mask = (tok + kTile > unmasked_end) || !row_ok || !tile_ok;
      const int lim = tile_ok ? vis_end : 0;

      // ---- S^T[token][row] = Kt * Qhat^T ----
      // These MFMAs accumulate in ordinary VGPRs (written as inline assembly) because all 256 accumulation
      // registers hold O^T; the compiler's own MFMA selection would put S^T there as well and spill.
      f32x16 s;
      // With few query rows the kernel is bound by how many bytes it keeps in flight, not by its MFMAs: the request
      // for tile it + kAhead goes out first (no LDS read is outstanding here either).
      if constexpr (SPLIT > 1) {
        if (stage_next) stage_panels_full<kTile, NP, 4, ROWB>(next_buf, next_g, wave, lane);
      }
      if constexpr (SPLIT == 1) {
        bf16x8 f[3][4];  // ring of fragment batches: loads run two batches (8 MFMAs) ahead of their use
#pragma unroll
        for (int b = 0; b < 4; ++b) f[0][b] = *(const bf16x8*)(buf + kbase[b]);
#pragma unroll
        for (int b = 0; b < 4; ++b) f[1][b] = *(const bf16x8*)(buf + kbase[b] + PANEL);
#pragma unroll
        for (int a4 = 0; a4 < KS / 4; ++a4) {
          if (a4 + 2 < KS / 4) {
#pragma unroll
            for (int b = 0; b < 4; ++b) f[(a4 + 2) % 3][b] = *(const bf16x8*)(buf + kbase[b] + ((a4 + 2) * PANEL));
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            if (a4 == 0 && b == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(f[0][0]), "v"(qf[0]));  // result registers must not overlap the operands
            else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(f[a4 % 3][b]), "v"(qf[4 * a4 + b]));
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
        bf16x8 f[KS / 4][KB];  // this wave's share is short: every fragment is requested up front
#pragma unroll
        for (int a4 = 0; a4 < KS / 4; ++a4)
#pragma unroll
          for (int b = 0; b < KB; ++b) f[a4][b] = *(const bf16x8*)(buf + kbase[b] + a4 * PANEL);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int a4 = 0; a4 < KS / 4; ++a4)
#pragma unroll
          for (int b = 0; b < KB; ++b) {
            if (a4 == 0 && b == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(f[0][0]), "v"(qf[0]));  // result registers must not overlap the operands
            else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(f[a4][b]), "v"(qf[a4 * KB + b]));
          }
        __builtin_amdgcn_sched_barrier(0);
      }
      // Tile it + kAhead is requested here, in one burst: at this point no LDS read of this wave is outstanding.
      // (An LDS-DMA instruction issued while reads are in flight holds the wave, and with it the MFMA stream, until
      // they have returned.)
      if constexpr (SPLIT == 1) {
        if (stage_next) stage_panels_full<kTile, NP, 4, ROWB>(next_buf, next_g, wave, lane);
      }
      // first batches of value fragments: issued now, consumed after the softmax
      i16x4 r[3][4][2];
      auto load_v = [&](int slot, int u, int p4) {  // output tiles dt = 4*p4 .. 4*p4 + 3 of k-step u
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const int dt = 4 * p4 + d;
          const int off = (dt >> 1) * PANEL + (16 * u) * 128;
          r[slot][d][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(buf + vbase + (off + 64 * (dt & 1))));
          r[slot][d][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(buf + vbase + (off + 8 * 128 + 64 * (1 - (dt & 1)))));
        }
      };
      constexpr int NBT = 2 * (DTW / 4);  // batches of four value fragments: k-step bt / (DTW/4), tiles 4*(bt % (DTW/4)) ..
      load_v(0, 0, 0);
      load_v(1, 1 / (DTW / 4), 1 % (DTW / 4));
      // the matrix pipeline's result is not interlocked against vector-ALU reads: wait out its 8 passes
      asm volatile("s_nop 15\n\ts_nop 7" : "+v"(s));
      if constexpr (SPLIT > 1) {
        // team sum of the partial S^T: [wave][quarter][lane] 16-byte slots behind the tile ring
        char* ex = smem + kSlots * TILE_BYTES;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          *(f32x4*)(ex + wave * 4096 + q * 1024 + lane * 16) = f32x4{s[4 * q], s[4 * q + 1], s[4 * q + 2], s[4 * q + 3]};
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
        __syncthreads();  // the next write to these slots comes after the next tile's barrier, which follows these reads
#pragma unroll
        for (int w = 0; w < SPLIT; ++w)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const f32x4 x = *(const f32x4*)(ex + (team * SPLIT + w) * 4096 + q * 1024 + lane * 16);
#pragma unroll
            for (int e = 0; e < 4; ++e) s[4 * q + e] = (w == 0) ? x[e] : s[4 * q + e] + x[e];
          }
      }

      // ---- online softmax (base 2); register i is token tok + 8*(i/4) + 4*h + i%4 ----
      // The maximum is taken on the raw logits (the scale is positive) and the scale rides in the exponent's FMA.
      if (__builtin_amdgcn_ballot_w64(need_mask) != 0) {  // wave-uniform: only tiles at the chunk end, or padding rows
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (need_mask && tok + 8 * (i >> 2) + 4 * h + (i & 3) >= lim) s[i] = GQLA_NEG_INF;
      }
      float tmax = s[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, s[i]);
      tmax = pair_max(tmax) * a.scale_log2e;
      if (__builtin_amdgcn_ballot_w64(tmax > m_ref + kRescaleThreshold) != 0) {
        const float m_new = fmaxf(m_ref, tmax);
        const float alpha = fast_exp2(m_ref - ((m_new == GQLA_NEG_INF) ? 0.f : m_new));
        m_ref = m_new;
        l_run *= alpha;
        if (it > 0) acc_scale(alpha);
      }
      const float m_use = (m_ref == GQLA_NEG_INF) ? 0.f : m_ref;
      // P^T fragments, k-step u: tokens 16*u + {4h..4h+3, 8+4h..8+4h+3}.  Only the first is finished before the
      // O^T update starts; the exponentials of the second ride in the shadow of the first k-step's MFMAs (one
      // exponential, its FMA and its add fit behind one MFMA of the same wave).
      bf16x8 pf[2];
      float p1[8];
      u32x4 w1;
      if constexpr (SPLIT > 1) {  // too few MFMAs per k-step to hide exponentials behind: both halves now
        float psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          p1[e] = fast_exp2(__builtin_fmaf(s[8 + e], a.scale_log2e, -m_use));
          psum += p1[e];
        }
        w1 = u32x4{pack_bf16(p1[0], p1[1]), pack_bf16(p1[2], p1[3]), pack_bf16(p1[4], p1[5]), pack_bf16(p1[6], p1[7])};
        l_run += psum;
      }
      {
        float p[8], psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          p[e] = fast_exp2(__builtin_fmaf(s[e], a.scale_log2e, -m_use));
          psum += p[e];
        }
        u32x4 w = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
        pf[0] = __builtin_bit_cast(bf16x8, w);
        l_run += psum;
      }
      // An MFMA may read a register as an operand no sooner than two wait states after a vector-ALU instruction wrote
      // it.  The compiler keeps that distance for its own MFMAs but does not look inside inline assembly, so the
      // distance between the last pack of the probabilities and the first O^T update is made here.
      if constexpr (SPLIT > 1) asm volatile("s_nop 1" : "+v"(pf[0]), "+v"(w1));
      else asm volatile("s_nop 1" : "+v"(pf[0]));
      __builtin_amdgcn_sched_barrier(0);

      // ---- O^T[r][row] += C^T * P^T, value fragments one batch of four tiles ahead ----
#pragma unroll
      for (int bt = 0; bt < NBT; ++bt) {
        const int u = bt / (DTW / 4), p4 = bt % (DTW / 4);
        if (bt + 2 < NBT) load_v((bt + 2) % 3, (bt + 2) / (DTW / 4), (bt + 2) % (DTW / 4));
        if (bt == DTW / 4) pf[1] = __builtin_bit_cast(bf16x8, w1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const i16x4 lo = r[bt % 3][d][0], hi = r[bt % 3][d][1];
          const i16x8 fr = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          acc_mfma(4 * p4 + d, __builtin_bit_cast(bf16x8, fr), pf[u]);
          if (SPLIT == 1 && u == 0) {  // second k-step's probabilities, one piece per MFMA
            const int idx = 4 * bt + d;
            if (idx < 8) {
              p1[idx] = fast_exp2(__builtin_fmaf(s[8 + idx], a.scale_log2e, -m_use));
              l_run += p1[idx];
            } else if (idx < 12) {
              w1[idx - 8] = pack_bf16(p1[2 * (idx - 8)], p1[2 * (idx - 8) + 1]);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    shift_pages();
  }

  const float l_tot = pair_sum(l_run);
  if (!row_ok) return;
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  const int64_t prow = (int64_t)chunk * a.M + rho;
  __bf16* po = (__bf16*)a.part_o + prow * RKV;
#pragma unroll
  for (int dt = 0; dt < DTW; ++dt) {
    float x[16];
    acc_read(dt, dt == 0, x);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      u32x2 v = {pack_bf16(x[4 * q] * inv, x[4 * q + 1] * inv), pack_bf16(x[4 * q + 2] * inv, x[4 * q + 3] * inv)};
      *(u32x2*)(po + (part * DTW + dt) * 32 + 8 * q + 4 * h) = v;
    }
  }
  if (h == 0 && part == 0) a.part_lse[prow] = l_tot > 0.f ? (m_ref + fast_log2(l_tot)) * kLn2 : GQLA_NEG_INF;
}

// ---- combine + latent-output projection: out = W_UV[j]^T (sum_k w_k o_hat_k)   (MQA-absorb equation, line 6) ----
// One workgroup of 4 waves per (group j, 32 query rows of that group; 8 rows when the batch is small).  W_UV[j] ([r_kv][d_h], 128 KB) is staged in LDS
// and read transposed; wave w contracts over latent dims [w*RKV/4, (w+1)*RKV/4):
//   O^T[d][row] += W^T[d][r] * Ohat^T[r][row]     A = transposed LDS fragments, B = the combined chunk partials
// and the four partial O^T are summed through LDS.
// DV: value dims per head (columns of W_UV[j], elements of an output row); a workgroup projects onto DH = 128 of them,
// blockIdx.z selects which (the staged slice of W_UV is then 128 KB whatever DV is; the merge is repeated per slice).
template <int RKV, int DH, int DV>
__global__ void __launch_bounds__(256) combine_project_bf16_kernel(CombineArgs a, int rows_per_group, int rows_per_wg) {
  constexpr int KSW = RKV / 16 / 4;  // k-steps per wave
  constexpr int MT = DH / 32;
  static_assert(MT == 4, "one output tile per wave in the final reduction");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 31, h = lane >> 5;
  const int j = blockIdx.y;
  const int col0 = blockIdx.z * DH;  // first value dim of this workgroup
  stage_panels_full<RKV, DH / 64, 4, DV * 2>(smem, (const char*)a.w_uv + ((int64_t)j * RKV * DV + col0) * 2, wave, lane);

  // row of this lane among the rows of group j: x = (b * s_q + t) * G + head-in-group
  // rows_per_wg < 32 (small batches): more workgroups, each with only its first lanes holding a row, so that the merge of
  // many chunk partials is spread over the chip; lanes without a row compute on row 0 and store nothing.
  const int x = blockIdx.x * rows_per_wg + n;
  const bool row_ok = n < rows_per_wg && x < rows_per_group;
  const int xc = row_ok ? x : 0;
  const int b = xc / (a.s_q * a.G);
  const int t = (xc / a.G) % a.s_q;
  const int rho = t * a.h_q + j * a.G + xc % a.G;
  const int s0 = a.first_slot[b], s1 = a.first_slot[b + 1];
  // Log-sum-exp merge of the row's chunk partials in ONE pass, kNB chunks at a time so that their loads (log-sum-exps
  // and latent vectors) are in flight together; the running maximum moves as in an online softmax.  (Three passes
  // with one dependent load per chunk each cost three memory latencies per chunk.)
  constexpr int kNB = 4;
  float m = GQLA_NEG_INF, den = 0.f;
  // combined latent output of this lane's row, dims 16*(KSW*wave + ksl) + 8*h + 0..7, fp32
  float acc[KSW][8];
#pragma unroll
  for (int ksl = 0; ksl < KSW; ++ksl)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[ksl][e] = 0.f;
  const __bf16* po = (const __bf16*)a.part_o + (int64_t)rho * RKV + (KSW * wave) * 16 + h * 8;
  for (int sb = s0; sb < s1; sb += kNB) {
    float l[kNB];
    u32x4 v[kNB][KSW];
#pragma unroll
    for (int k = 0; k < kNB; ++k) {
      const int sc = min(sb + k, s1 - 1);  // clamped: a chunk beyond the range is loaded again and given weight 0
      l[k] = a.part_lse[(int64_t)sc * a.M + rho];
#pragma unroll
      for (int ksl = 0; ksl < KSW; ++ksl) v[k][ksl] = *(const u32x4*)(po + (int64_t)sc * a.M * RKV + ksl * 16);
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
    for (int ksl = 0; ksl < KSW; ++ksl)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[ksl][e] *= rescale;
    m = m_new;
#pragma unroll
    for (int k = 0; k < kNB; ++k) {
      const float w = __expf(l[k] - m_use);
      den += w;
#pragma unroll
      for (int ksl = 0; ksl < KSW; ++ksl)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[ksl][2 * e] += w * bf16_bits_to_float(v[k][ksl][e] & 0xffffu);
          acc[ksl][2 * e + 1] += w * bf16_bits_to_float(v[k][ksl][e] >> 16);
        }
    }
  }
  const float inv_den = (row_ok && den > 0.f) ? 1.f / den : 0.f;
#pragma unroll
  for (int ksl = 0; ksl < KSW; ++ksl)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[ksl][e] *= inv_den;

  wait_all_memory();
  __syncthreads();  // W_UV[j] staged

  const TrNatural tr = make_tr_natural(lane);
  f32x16 o[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[mt][i] = 0.f;
  const char* wbase = smem + (KSW * wave) * 2048;  // this wave's rows of the staged matrix
#pragma unroll
  for (int ksl = 0; ksl < KSW; ++ksl) {
    u32x4 pw = {pack_bf16(acc[ksl][0], acc[ksl][1]), pack_bf16(acc[ksl][2], acc[ksl][3]),
                pack_bf16(acc[ksl][4], acc[ksl][5]), pack_bf16(acc[ksl][6], acc[ksl][7])};
    const bf16x8 bfrag = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) o[mt] = mfma32(tr_natural_frag<RKV>(wbase, tr, ksl, mt), bfrag, o[mt]);
  }

  // sum the four waves' partial O^T through LDS: slot [wave][mt][i][lane]
  __syncthreads();  // everyone is done reading the staged weights
  float* red = (float*)smem;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) red[((wave * MT + mt) * 16 + i) * 64 + lane] = o[mt][i];
  __syncthreads();
  float r[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    r[i] = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) r[i] += red[((w * MT + wave) * 16 + i) * 64 + lane];
  }
  if (!row_ok) return;
  __bf16* out = (__bf16*)a.out + ((int64_t)b * a.M + rho) * DV + col0 + wave * 32;  // this wave writes dims col0 + 32*wave .. +31
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    u32x2 v = {pack_bf16(r[4 * q], r[4 * q + 1]), pack_bf16(r[4 * q + 2], r[4 * q + 3])};
    *(u32x2*)(out + 8 * q + 4 * h) = v;
  }
  if (a.lse && h == 0 && wave == 0 && col0 == 0) a.lse[(int64_t)b * a.M + rho] = m + __logf(den);
}

}  // namespace

template <int SPLIT>
static hipError_t launch_decode_absorb_split(const DecodeArgs& a, hipStream_t s) {
  // tile ring, plus the team exchange (4 KB per wave) when waves share rows
  constexpr int kLds = kSlots * kTile * (512 + 64) * 2 + (SPLIT > 1 ? 4 * 4096 : 0);
  // once per process (function-local statics are initialised under a lock); an error is reported by every call
  static const hipError_t attr =
      hipFuncSetAttribute((const void*)decode_absorb_bf16_kernel<512, 64, SPLIT>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
  if (attr != hipSuccess) return attr;
  const int row_blocks = (a.M + kRowsPerBlock / SPLIT - 1) / (kRowsPerBlock / SPLIT);
  const int chunks_padded = (a.n_chunks + 7) / 8 * 8;
  decode_absorb_bf16_kernel<512, 64, SPLIT><<<chunks_padded * row_blocks, 256, kLds, s>>>(a, row_blocks);
  return hipGetLastError();
}

hipError_t launch_decode_absorb_bf16(const DecodeArgs& a, hipStream_t s) {
  // At most 32 query rows: the four waves share them, so that none is left without work.  More rows but few chunks
  // (small batches): one workgroup per (chunk, 32 rows) with the four waves sharing its rows, as long as all of them
  // still run at once -- four times the workgroups, each with a shorter tile (the tiles' re-reads hit the L2, and
  // with so few chunks the chip is nowhere near its memory rate).
  const int chunks_padded = (a.n_chunks + 7) / 8 * 8;
  if (a.M <= 32 || chunks_padded * ((a.M + 31) / 32) <= a.num_cus) return launch_decode_absorb_split<4>(a, s);
  return launch_decode_absorb_split<1>(a, s);
}

template <int DV>
static hipError_t launch_combine_project_dv(const CombineArgs& a, hipStream_t s) {
  constexpr int kLds = 512 * 128 * 2;
  // once per process (function-local statics are initialised under a lock); an error is reported by every call
  static const hipError_t attr =
      hipFuncSetAttribute((const void*)combine_project_bf16_kernel<512, 128, DV>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
  if (attr != hipSuccess) return attr;
  const int rows_per_group = a.B * a.s_q * a.G;
  // 32 rows per workgroup fill the MFMA tile; with fewer than half a chip's worth of such workgroups, 8 or 4 rows each
  const int rows_per_wg = ((rows_per_group + 31) / 32) * a.g >= 128 ? 32 : (((rows_per_group + 7) / 8) * a.g >= 128 ? 8 : 4);
  combine_project_bf16_kernel<512, 128, DV><<<dim3((rows_per_group + rows_per_wg - 1) / rows_per_wg, a.g, DV / 128), 256, kLds, s>>>(
      a, rows_per_group, rows_per_wg);
  return hipGetLastError();
}

hipError_t launch_combine_project_bf16(const CombineArgs& a, hipStream_t s) {
  return a.d_h == 256 ? launch_combine_project_dv<256>(a, s) : launch_combine_project_dv<128>(a, s);  // a.d_h: value dims here
}

}  // namespace gqla
