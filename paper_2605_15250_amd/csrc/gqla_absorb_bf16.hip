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
#include <cstdlib>
#include <type_traits>
#include <utility>

#include "gqla_device.h"
#include "gqla_lds.h"

#ifdef GQLA_PHASE_TIMING
__device__ unsigned long long gqla_phase_cycles[16];
extern "C" int gqla_debug_read_phases(unsigned long long* host16, int reset) {
  if (hipMemcpyFromSymbol(host16, HIP_SYMBOL(gqla_phase_cycles), 16 * 8) != hipSuccess) return 1;
  if (reset) {
    unsigned long long z[16] = {};
    if (hipMemcpyToSymbol(HIP_SYMBOL(gqla_phase_cycles), z, 16 * 8) != hipSuccess) return 1;
  }
  return 0;
}
#if GQLA_PHASE_TIMING >= 2
#define GQLA_STAMP(k) do { const long long now_ = __builtin_readcyclecounter(); ph_[k] += now_ - last_; last_ = now_; } while (0)
#else
#define GQLA_STAMP(k) do { (void)ph_; (void)last_; } while (0)   // level 1: kernel entry and exit only
#endif
#else
#define GQLA_STAMP(k) do { } while (0)
#endif

namespace gqla {

namespace {

__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

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
#define GQLA_ACC_CLOBBER(D) GQLA_ACC_CLOBBER_##D
#define GQLA_ACC_CLOBBER_0 "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15"
#define GQLA_ACC_CLOBBER_1 "a16", "a17", "a18", "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31"
#define GQLA_ACC_CLOBBER_2 "a32", "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", "a45", "a46", "a47"
#define GQLA_ACC_CLOBBER_3 "a48", "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", "a58", "a59", "a60", "a61", "a62", "a63"
#define GQLA_ACC_CLOBBER_4 "a64", "a65", "a66", "a67", "a68", "a69", "a70", "a71", "a72", "a73", "a74", "a75", "a76", "a77", "a78", "a79"
#define GQLA_ACC_CLOBBER_5 "a80", "a81", "a82", "a83", "a84", "a85", "a86", "a87", "a88", "a89", "a90", "a91", "a92", "a93", "a94", "a95"
#define GQLA_ACC_CLOBBER_6 "a96", "a97", "a98", "a99", "a100", "a101", "a102", "a103", "a104", "a105", "a106", "a107", "a108", "a109", "a110", "a111"
#define GQLA_ACC_CLOBBER_7 "a112", "a113", "a114", "a115", "a116", "a117", "a118", "a119", "a120", "a121", "a122", "a123", "a124", "a125", "a126", "a127"
#define GQLA_ACC_CLOBBER_8 "a128", "a129", "a130", "a131", "a132", "a133", "a134", "a135", "a136", "a137", "a138", "a139", "a140", "a141", "a142", "a143"
#define GQLA_ACC_CLOBBER_9 "a144", "a145", "a146", "a147", "a148", "a149", "a150", "a151", "a152", "a153", "a154", "a155", "a156", "a157", "a158", "a159"
#define GQLA_ACC_CLOBBER_10 "a160", "a161", "a162", "a163", "a164", "a165", "a166", "a167", "a168", "a169", "a170", "a171", "a172", "a173", "a174", "a175"
#define GQLA_ACC_CLOBBER_11 "a176", "a177", "a178", "a179", "a180", "a181", "a182", "a183", "a184", "a185", "a186", "a187", "a188", "a189", "a190", "a191"
#define GQLA_ACC_CLOBBER_12 "a192", "a193", "a194", "a195", "a196", "a197", "a198", "a199", "a200", "a201", "a202", "a203", "a204", "a205", "a206", "a207"
#define GQLA_ACC_CLOBBER_13 "a208", "a209", "a210", "a211", "a212", "a213", "a214", "a215", "a216", "a217", "a218", "a219", "a220", "a221", "a222", "a223"
#define GQLA_ACC_CLOBBER_14 "a224", "a225", "a226", "a227", "a228", "a229", "a230", "a231", "a232", "a233", "a234", "a235", "a236", "a237", "a238", "a239"
#define GQLA_ACC_CLOBBER_15 "a240", "a241", "a242", "a243", "a244", "a245", "a246", "a247", "a248", "a249", "a250", "a251", "a252", "a253", "a254", "a255"
#define GQLA_FOR_DT(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15)

__device__ __forceinline__ void acc_zero() {
  asm volatile(".set gqla_i, 0\n.rept 256\n\tv_accvgpr_write_b32 a[gqla_i], 0\n.set gqla_i, gqla_i+1\n.endr" : : : GQLA_ALL_AGPRS);
}
// O^T tile dt += A * B (dt is a compile-time value at every call site: the switch folds away)
__device__ __forceinline__ void acc_mfma(int dt, bf16x8 a, bf16x8 b) {
  switch (dt) {
    // (the tile's registers are named as clobbered: the compiler must not keep values of its own in them across this
    // statement -- it would otherwise use "free" accumulation registers as parking space when ordinary ones run short)
#define X(D) case D: asm volatile("v_mfma_f32_32x32x16_bf16 " GQLA_ACC(D) ", %0, %1, " GQLA_ACC(D) : : "v"(a), "v"(b) : GQLA_ACC_CLOBBER(D)); break;
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
  stage_panels_full<kTile, NP, 4, ROWB, true>(smem, tile_src(pg0, 0), wave, lane);
  if (n_tiles > 1) stage_panels_full<kTile, NP, 4, ROWB, true>(smem + TILE_BYTES, tile_src(pg1, kTile % P), wave, lane);
  if (n_tiles > 2) stage_panels_full<kTile, NP, 4, ROWB, true>(smem + 2 * TILE_BYTES, tile_src(pg2, (2 * kTile) % P), wave, lane);

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
      if (stage_next) stage_panels_full<kTile, NP, 4, ROWB, true>(next_buf, next_g, wave, lane);
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
        if (stage_next) stage_panels_full<kTile, NP, 4, ROWB, true>(next_buf, next_g, wave, lane);
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
        if (stage_next) stage_panels_full<kTile, NP, 4, ROWB, true>(next_buf, next_g, wave, lane);
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
  // this lane holds dims 4 h .. 4 h + 3 of vector 4 (part DTW + dt) + q of its row: with consecutive rows in consecutive
  // lanes a store instruction writes 512 contiguous bytes
  __bf16* po = (__bf16*)a.part_o + part_vec_index(chunk, rho, a.M, RKV / 8, 0) * 8 + 4 * h;
#pragma unroll
  for (int dt = 0; dt < DTW; ++dt) {
    float x[16];
    acc_read(dt, dt == 0, x);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      u32x2 v = {pack_bf16(x[4 * q] * inv, x[4 * q + 1] * inv), pack_bf16(x[4 * q + 2] * inv, x[4 * q + 3] * inv)};
      *(u32x2*)(po + ((part * DTW + dt) * 4 + q) * (32 * 8)) = v;
    }
  }
  if (h == 0 && part == 0) a.part_lse[prow] = l_tot > 0.f ? (m_ref + fast_log2(l_tot)) * kLn2 : GQLA_NEG_INF;
}

// every accumulator of row block rb (tiles 4*dtl + rb, dtl = 0..3) of this lane times alpha
__device__ __forceinline__ void acc_scale_rb(int rb, float alpha) {
  float t0, t1;
  switch (rb) {
#define X(R)                                                                                                             \
  case R:                                                                                                                \
    asm volatile(".irp gqla_t, " #R ", 4+" #R ", 8+" #R ", 12+" #R "\n.set gqla_i, 0\n.rept 8\n"                          \
                 "\tv_accvgpr_read_b32 %0, a[(\\gqla_t)*16+gqla_i]\n\tv_accvgpr_read_b32 %1, a[(\\gqla_t)*16+gqla_i+1]\n"  \
                 "\tv_mul_f32 %0, %0, %2\n\tv_mul_f32 %1, %1, %2\n\ts_nop 0\n"                                              \
                 "\tv_accvgpr_write_b32 a[(\\gqla_t)*16+gqla_i], %0\n\tv_accvgpr_write_b32 a[(\\gqla_t)*16+gqla_i+1], %1\n" \
                 ".set gqla_i, gqla_i+2\n.endr\n.endr"                                                                     \
                 : "=&v"(t0), "=&v"(t1)                                                                                    \
                 : "v"(alpha));                                                                                            \
    break;
    X(0) X(1) X(2) X(3)
#undef X
  }
}

// More than 32 query rows per sequence and enough chunks to fill the chip: one workgroup of 4 waves per (chunk, block of
// 128 rows), and the two contractions are dealt over the waves in two different ways.
//   S^T: wave w owns row block w (rows 32w..32w+31) against the whole tile, queries in registers.
//   O^T: wave w owns latent dims 128w..128w+127 of ALL four row blocks: accumulator tile 4*d + rb holds dims
//        128w + 32d.. of row block rb.  Each transposed value fragment read from LDS then feeds four MFMAs (one per row
//        block) instead of one, which cuts the transposed reads per tile by four; the price is that the waves trade
//        their probabilities: wave rb writes its two P^T operand fragments (1 KB each, already in B-operand order) into a
//        double-buffered 8 KB exchange behind the tile ring, and every wave reads all eight.
// The loop is software-pipelined so that nothing but MFMAs (and what fits in their shadows) is on a wave's critical path
// (measured on this chip: behind each 32-cycle MFMA a wave issues four simple vector-ALU instructions or two
// exponentials for free, an LDS read costs about 5 cycles, an LDS-DMA instruction 10-20):
//   iteration i:   S^T(i)          36 MFMAs; in their gaps: the key-fragment reads (a ring of 8 fragments, 8 MFMAs ahead),
//                                  the 9 LDS-DMA instructions that stage tile i+2, and the first operands of the next phase
//                  O^T += (i-1)    32 MFMAs; in their gaps: the softmax of tile i (maximum, exponentials, packing) and the
//                                  write of its probabilities
//                  one workgroup barrier, then the first key fragments of tile i+1 are requested
// The barrier is the only one of the tile: each wave waits for its share of tile i+1's staging before it arrives, so
// passing it means "tile i+1 has landed for everyone", "the probabilities of tile i are visible" and "everyone is done
// with tile i-1", whose buffer the staging of tile i+3 (issued in the next iteration's gaps) overwrites.
// The softmax state (reference maximum, denominator) of a row lives in the wave that owns its row block.  A move of the
// reference maximum of rows that already have output (rare: the maximum must grow by more than 2^8) has to rescale
// accumulators in all four waves: the owning wave announces it in the sign bit of its first probability (probabilities
// are never negative), all waves see the same bits, and together they take a slow path that passes the factors through
// the idle half of the exchange.
// Requires whole blocks of 128 rows (h_q s_q a multiple of 128; the launcher sends other row counts to the kernel above):
// there is no branch per row block, and the register budget is exact -- the compiler must never run out of ordinary
// registers here, or it would park values in accumulation registers, which hold O^T behind its back (the MFMA
// statements name their accumulators as clobbered, and the build checks the generated code for both).
template <int RKV, int DR>
__global__ void __launch_bounds__(256) decode_absorb_shared_bf16_kernel(DecodeArgs a, int row_blocks) {
  constexpr int W = RKV + DR;
  constexpr int ROWB = W * 2;
  constexpr int NP = W / 64;
  constexpr int PANEL = kTile * 128;
  constexpr int KS = W / 16;
  constexpr int DT = RKV / 32;
  constexpr int TILE_BYTES = kTile * ROWB;
  constexpr int EX = kSlots * TILE_BYTES;  // exchange: [2 buffers][4 row blocks][2 k-steps][64 lanes][16 bytes]
  constexpr int KR = 4;                    // key fragments in flight (more do not fit the 256 ordinary registers)
  static_assert(DT == 16, "O^T fills the 256 accumulation registers exactly: 4 dim tiles x 4 row blocks per wave");
  static_assert(W % 64 == 0 && RKV % 128 == 0, "latent row must be a whole number of 128-byte panels, two per wave");
  static_assert(KS == 36 && NP == 9, "the gap schedule below is written for 36 key k-steps and 9 staging instructions");
  extern __shared__ __attribute__((aligned(16))) char smem[];

  int chunk, rbk;
  {
    const int id = blockIdx.x;
    const int grp = id / (8 * row_blocks), rem = id % (8 * row_blocks);
    rbk = rem / 8;
    chunk = grp * 8 + rem % 8;
  }
  if (chunk >= a.n_chunks) return;  // whole workgroup leaves together
#ifdef GQLA_PHASE_TIMING
  const long long t_entry_ = __builtin_readcyclecounter();
  long long ph_[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  long long last_ = t_entry_;
#endif
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 31, h = lane >> 5;
  const ChunkEntry ce = a.chunks[chunk];

  const int row0 = rbk * kRowsPerBlock;
  const int rho = row0 + wave * 32 + n;  // row = t * h_q + i (always a real row here)
  const int t = rho / a.h_q;
  const int vis_end = min(ce.tok_end, ce.L - a.s_q + t + 1);
  const int unmasked_end = min(ce.tok_end, ce.L - a.s_q + 1);

  const int P = a.cache.page_size;
  const char* pool = (const char*)a.cache.pool;
  const int32_t* table_row = a.cache.page_table ? a.cache.page_table + (int64_t)ce.b * a.cache.max_pages : nullptr;
  auto checked = [&](int32_t pg) -> int32_t { return ((uint32_t)pg < (uint32_t)a.cache.num_pages) ? pg : -1; };
  auto tile_src = [&](int32_t pg, int slot) -> const char* { return pool + ((int64_t)(pg >= 0 ? pg : 0) * P + slot) * ROWB; };

  // per-lane LDS offsets inside a tile (panel layout of gqla_lds.h): key fragment of k-step ks = 4*a4 + b at
  // kbase[b] + a4*PANEL; transposed value reads at vbase + compile-time offsets (this wave's dims: panels 2w, 2w+1)
  uint32_t kbase[4], vbase;
  {
#pragma unroll
    for (int b = 0; b < 4; ++b) kbase[b] = n * 128 + (((2 * b + h) ^ lds_swz(n)) << 4);
    const int i16 = lane & 15, e = i16 >> 2, q = i16 & 3, g1 = (lane >> 4) & 1;
    vbase = (4 * h + e) * 128 + (((2 * g1 + (q >> 1)) ^ (2 * h + (e >> 1))) << 4) + (q & 1) * 8;
    vbase += wave * 2 * PANEL;
  }
  const uint32_t stage_off = stage_lane_offset<kTile, NP, 4, ROWB>(wave, lane);

  GQLA_STAMP(4);
  float m_ref = GQLA_NEG_INF, l_run = 0.f;

  // the queries are requested first: their addresses need only the chunk entry, and they are the bulk of what a
  // workgroup waits for before its first MFMA; the page ids (a dependent scalar load) arrive in their shadow
  bf16x8 qf[KS];
  {
    const int64_t qrow = (int64_t)ce.b * a.M + rho;
    const __bf16* ph = (const __bf16*)a.q_a + qrow * RKV + h * 8;
    const __bf16* pr = (const __bf16*)a.q_r + qrow * DR + h * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8*)(ks < RKV / 16 ? ph + ks * 16 : pr + (ks - RKV / 16) * 16);
  }

  const int n_tiles = (ce.tok_end - ce.tok_begin + kTile - 1) / kTile;
  // page ids of tiles it .. it+3; iteration `it` stages tile it+2 (the first three are staged up front), the table entry
  // of tile it+4 travels through the scalar cache meanwhile
  int32_t pg0, pg1, pg2, pg3;
  {
    const int p_last = (ce.tok_end - 1) / P;
    int32_t raw[4];
    if (table_row) {
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
  GQLA_STAMP(5);
  int32_t pg_raw = 0;
  const char* next_g = pool;  // first row of the tile the next iteration stages (set when the window moves)
  const int p_first = ce.tok_begin / P;
  int st_slot = (3 * kTile) % P;                                     // slot of tile it+3 in its page
  int lk_slot = (4 * kTile) % P, lk_p = p_first + (4 * kTile) / P;   // tile it+4

  // Start-up: all workgroups begin at once, on cold address translations, and each walks a chain of dependent first
  // touches (chunk entry, page table, queries and tile 0): about 15 k cycles pass before the first MFMA, 7 % of the
  // kernel at the canonical shape, the same whether the queries (147 KB per workgroup, 38 MB over the chip) are loaded
  // as fragments or staged through LDS in whole lines, and the same with the chunks of a sequence on one die -- it is
  // neither the shape of the loads nor their volume.  The queries go first (above), then tile 0; tiles 1 and 2 are
  // requested once those have landed, while tile 0 is being multiplied.
  stage_panels_full<kTile, NP, 4, ROWB, true>(smem, tile_src(pg0, 0), wave, lane);
  acc_zero();  // 256 register writes, in the shadow of the requests above
  // The query loads complete here, before the loop (the compiler's wait for them also covers the request for tile 0
  // above); inside the loop only hand-counted waits remain.
#pragma unroll
  for (int k = 0; k < KS; k += 9)
    asm volatile("" : "+v"(qf[k]), "+v"(qf[k + 1]), "+v"(qf[k + 2]), "+v"(qf[k + 3]), "+v"(qf[k + 4]), "+v"(qf[k + 5]),
                      "+v"(qf[k + 6]), "+v"(qf[k + 7]), "+v"(qf[k + 8]));

  // rows of a tile past the chunk end (or a whole tile behind an out-of-pool page id) hold whatever the page holds:
  // zeroed in LDS by the whole workgroup before anyone reads them, so that 0 * v stays 0
  auto zero_rows = [&](int slot, int valid) {
    for (int idx = threadIdx.x; idx < (kTile - valid) * (W / 8); idx += 256) {
      const int r = valid + idx / (W / 8), c = idx % (W / 8);
      *(u32x4*)(smem + slot * TILE_BYTES + (c >> 3) * PANEL + r * 128 + (c & 7) * 16) = u32x4{0u, 0u, 0u, 0u};
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
    __syncthreads();
  };
  GQLA_STAMP(6);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();  // the first tiles have landed for every wave
  GQLA_STAMP(7);
  if (n_tiles > 1) stage_panels_full<kTile, NP, 4, ROWB, true>(smem + TILE_BYTES, tile_src(pg1, kTile % P), wave, lane);
  if (n_tiles > 2) stage_panels_full<kTile, NP, 4, ROWB, true>(smem + 2 * TILE_BYTES, tile_src(pg2, (2 * kTile) % P), wave, lane);
  {
    const int valid0 = pg0 >= 0 ? min(kTile, ce.tok_end - ce.tok_begin) : 0;
    if (valid0 < kTile) zero_rows(0, valid0);
  }

  // operands that live across the phases of the pipeline
  bf16x8 kf[KR];        // key fragments, requested KR MFMAs ahead of their use
  bf16x8 pfr[4][2];     // probabilities of the tile whose O^T update is running: [row block][k-step]
  i16x4 vr[2][4][2];    // its value fragments [k-step][dim tile][read]
  f32x16 s;             // raw logits of the tile whose softmax is running
  float alpha_prev = 1.f;   // factor of this wave's rows announced with the probabilities of the previous tile
  bool announce_prev = false;

  auto load_k = [&](const char* tb, int ks) __attribute__((always_inline)) {  // key fragment of k-step ks of the tile at tb
    kf[ks % KR] = *(const bf16x8*)(tb + kbase[ks & 3] + (ks >> 2) * PANEL);
  };
  auto load_v = [&](const char* tb, int u, int d) __attribute__((always_inline)) {
    const int off = (d >> 1) * PANEL + (16 * u) * 128;
    vr[u][d][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(tb + vbase + (off + 64 * (d & 1))));
    vr[u][d][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(tb + vbase + (off + 8 * 128 + 64 * (1 - (d & 1)))));
  };
  auto load_p = [&](const char* exr, int rb, int u) __attribute__((always_inline)) { pfr[rb][u] = *(const bf16x8*)(exr + (rb * 2 + u) * 1024); };

#pragma unroll
  for (int ks = 0; ks < KR; ++ks) load_k(smem, ks);

  // Iterations 0 .. n_tiles: iteration it computes S^T of tile it (HAS_S: it < n_tiles) and updates O^T with tile it-1
  // (HAS_PV: it > 0); STAGE: tile it+2 exists and is staged in this iteration (tiles 0..2 were staged up front).  The
  // three flags are compile-time so that the steady-state body has no branch per gap.
  auto iteration = [&](int it, auto HAS_S_T, auto HAS_PV_T, auto STAGE_T) __attribute__((always_inline)) {
    constexpr bool HAS_S = decltype(HAS_S_T)::value, HAS_PV = decltype(HAS_PV_T)::value, STAGE = decltype(STAGE_T)::value;
    const int tok = ce.tok_begin + it * kTile;
    const char* buf = smem + (it & (kSlots - 1)) * TILE_BYTES;                 // tile it
    const char* pbuf = smem + ((it + kSlots - 1) & (kSlots - 1)) * TILE_BYTES;  // tile it-1
    const char* exr = smem + EX + ((it + 1) & 1) * 8192 + lane * 16;           // probabilities of tile it-1
    char* exw = smem + EX + (it & 1) * 8192;                                   // probabilities of tile it
    char* next_buf = smem + ((it + 2) & (kSlots - 1)) * TILE_BYTES;
    const bool lookup = it + 4 < n_tiles;
    const bool new_page = lookup && lk_slot == 0;
    if (new_page && table_row)  // scalar load, consumed at the end of the iteration (its wait is written out there)
      asm volatile("s_load_dword %0, %1, 0x0" : "=s"(pg_raw) : "s"(table_row + lk_p) : "memory");
    const bool tile_ok = pg0 >= 0;
    const int lk_p_prev = lk_p;
    // Tile it+1 becomes current: the window of page ids moves, and the source of the tile that the next iteration
    // stages (tile it+3) is formed.  Scalar work; it runs in the shadow of the first MFMA of phase 2.
    auto move_window = [&]() __attribute__((always_inline)) {
      pg0 = pg1;
      pg1 = pg2;
      pg2 = pg3;  // pg3 (tile it+4) is the same page unless a new one was looked up; set behind the barrier
      next_g = tile_src(pg2, st_slot);
      st_slot = lk_slot;
      lk_slot += kTile;
      if (lk_slot == P) {
        lk_slot = 0;
        ++lk_p;
      }
    };

    // ---------------- phase 1: S^T(it), staging of tile it+2, first operands of phase 2 ----------------
    if constexpr (HAS_S) {
      static_for<KS>([&](auto KSI) __attribute__((always_inline)) {
        constexpr int ks = decltype(KSI)::value;
        if (ks == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(kf[0]), "v"(qf[0]));
        else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(kf[ks % KR]), "v"(qf[ks]));
        __builtin_amdgcn_sched_barrier(0);
        if (ks + KR < KS) load_k(buf, ks + KR);
        if (STAGE && ks % 3 == 1 && ks / 3 < 9) stage_panels_step<kTile, NP, 4, ROWB, true>(next_buf, next_g, wave, stage_off, ks / 3);
        if (HAS_PV) {  // operands of the first k-step of the O^T update, in the last gaps
          if (ks >= 28 && ks < 32) load_p(exr, ks - 28, 0);
          if (ks >= 32) load_v(pbuf, 0, ks - 32);
        }
        __builtin_amdgcn_sched_barrier(0);
      });
    } else {  // the last iteration: only the O^T update of the last tile is left
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) load_p(exr, rb, 0);
#pragma unroll
      for (int d = 0; d < 4; ++d) load_v(pbuf, 0, d);
    }
    GQLA_STAMP(0);

    // ---------------- phase 2: O^T += tile it-1, softmax of tile it in the gaps ----------------
    if (HAS_PV) {
      // announced moves of the reference maximum (uniform over the workgroup: every wave sees the same bits)
      uint32_t flags = 0;
#pragma unroll
      for (int rb = 0; rb < 4; ++rb)
        flags |= __builtin_bit_cast(u32x4, pfr[rb][0])[0];
      if (__builtin_amdgcn_readfirstlane(flags & 0x8000u) != 0) {
        // the factors travel through the idle half of the exchange (no probabilities of tile it are written before the
        // second barrier below)
        float* al = (float*)exw;
        if (announce_prev) al[wave * 32 + n] = alpha_prev;  // both half-waves hold the row's factor and write the same value
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __syncthreads();
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
          u32x4 w = __builtin_bit_cast(u32x4, pfr[rb][0]);
          if (__builtin_amdgcn_readfirstlane(w[0] & 0x8000u) != 0) {
            acc_scale_rb(rb, al[rb * 32 + n]);
            w[0] &= ~0x8000u;
            pfr[rb][0] = __builtin_bit_cast(bf16x8, w);
          }
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __syncthreads();
      }
    }
    // softmax state of this iteration (pieces run in the gaps below)
    constexpr bool sm = HAS_S;
    const bool need_mask = (tok + kTile > unmasked_end) || !tile_ok;
    const int lim = tile_ok ? vis_end : 0;
    float tmax = 0.f, m_use = 0.f, psum = 0.f, alpha = 1.f;
    bool announce = false;
    u32x4 w0 = {0u, 0u, 0u, 0u}, w1 = {0u, 0u, 0u, 0u};
    auto softmax_piece = [&](auto GI) __attribute__((always_inline)) {  // g = 0..31: position in the phase
      constexpr int g = decltype(GI)::value;
      if (g == 2) {
        // S^T is read here for the first time: three MFMAs of the O^T update have been issued since its last MFMA, which
        // has therefore retired (the matrix pipeline's result is not interlocked against vector-ALU reads)
        if (__builtin_amdgcn_ballot_w64(need_mask) != 0) {  // wave-uniform: only tiles at the chunk end, or padding rows
          // register i is token tok + 4h + 8*(i/4) + i%4: compared as a constant against one per-lane distance (formed
          // here, so that no per-register offsets are kept alive across the loop)
          int dist = lim - tok - 4 * h;
          asm volatile("" : "+v"(dist));
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (need_mask && 8 * (i >> 2) + (i & 3) >= dist) s[i] = GQLA_NEG_INF;
        }
        // the row maximum of the tile: eight three-way maxima (written as instructions: the logits come out of inline
        // assembly, and the compiler would first canonicalise every one of them)
        tmax = max3(s[0], s[1], s[2]);
        tmax = max3(tmax, s[3], s[4]);
      } else if (g == 3) {
        tmax = max3(tmax, s[5], s[6]);
        tmax = max3(tmax, s[7], s[8]);
      } else if (g == 4) {
        tmax = max3(tmax, s[9], s[10]);
        tmax = max3(tmax, s[11], s[12]);
      } else if (g == 5) {
        tmax = max3(tmax, s[13], s[14]);
        tmax = max3(tmax, s[15], s[15]);
      } else if (g == 6) {
        tmax = pair_max(tmax) * a.scale_log2e;
        if (__builtin_amdgcn_ballot_w64(tmax > m_ref + kRescaleThreshold) != 0) {
          const float m_new = fmaxf(m_ref, tmax);
          alpha = fast_exp2(m_ref - ((m_new == GQLA_NEG_INF) ? 0.f : m_new));
          // a row whose maximum was -inf has seen no token yet: its accumulators are zero and need no factor
          announce = __builtin_amdgcn_ballot_w64(m_new != m_ref && m_ref != GQLA_NEG_INF) != 0;
          m_ref = m_new;
          l_run *= alpha;
        }
        m_use = (m_ref == GQLA_NEG_INF) ? 0.f : m_ref;
      } else if (g >= 7 && g < 23) {
        constexpr int e = g >= 7 && g < 23 ? g - 7 : 0;
        s[e] = fast_exp2(__builtin_fmaf(s[e], a.scale_log2e, -m_use));  // the probability replaces the logit
        psum += s[e];
      } else if (g >= 23 && g < 27) {
        constexpr int q = g >= 23 && g < 27 ? g - 23 : 0;
        w0[q] = pack_bf16(s[2 * q], s[2 * q + 1]);
        w1[q] = pack_bf16(s[8 + 2 * q], s[8 + 2 * q + 1]);
      } else if (g == 27) {
        l_run += psum;
        if (announce) w0[0] |= 0x8000u;  // sign bit of the first probability
        *(u32x4*)(exw + (wave * 2 + 0) * 1024 + lane * 16) = w0;
      } else if (g == 28) {
        *(u32x4*)(exw + (wave * 2 + 1) * 1024 + lane * 16) = w1;
      }
    };
    if (HAS_PV) {
      static_for<32>([&](auto GI) __attribute__((always_inline)) {
        constexpr int g = decltype(GI)::value;
        constexpr int u = g >> 4, d = (g >> 2) & 3, rb = g & 3;
        {
          const i16x4 lo = vr[u][d][0], hi = vr[u][d][1];
          const i16x8 fr = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          acc_mfma(4 * d + rb, __builtin_bit_cast(bf16x8, fr), pfr[rb][u]);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (g == 0 && HAS_S) move_window();
        if (g >= 8 && g < 12) load_p(exr, g - 8, 1);  // second k-step's operands, as the first k-step's registers free up
        if (g >= 12 && g < 16) load_v(pbuf, 1, g - 12);
        if (sm) softmax_piece(GI);
        __builtin_amdgcn_sched_barrier(0);
      });
    } else {  // the first iteration: there is no O^T update yet to hide the softmax behind
      move_window();
      asm volatile("s_nop 15\n\ts_nop 7" : "+v"(s));  // the matrix pipeline's result is not interlocked against vector-ALU reads
      static_for<32>([&](auto GI) __attribute__((always_inline)) { softmax_piece(GI); });
    }
    alpha_prev = alpha;
    announce_prev = announce;
    GQLA_STAMP(1);

    // ---------------- the tile's barrier ----------------
    if (HAS_S) {
      if (it + 2 < n_tiles) asm volatile("s_waitcnt vmcnt(9)" ::: "memory");  // this wave's share of tile it+1 has landed
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the probabilities are written
      __syncthreads();
      GQLA_STAMP(2);
      if (it + 1 < n_tiles) {
        const int valid1 = pg0 >= 0 ? min(kTile, ce.tok_end - (tok + kTile)) : 0;  // (the window has moved: pg0 is tile it+1)
        if (valid1 < kTile) zero_rows((it + 1) & (kSlots - 1), valid1);  // only the chunk's last tile can have invalid rows
        const char* nbuf = smem + ((it + 1) & (kSlots - 1)) * TILE_BYTES;
#pragma unroll
        for (int ks = 0; ks < KR; ++ks) load_k(nbuf, ks);
      }
      // the page of tile it+4 joins the window (the scalar load was requested at the top of the iteration; no LDS
      // operation is outstanding here, so its wait costs nothing extra)
      if (new_page && table_row) asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(pg_raw) : : "memory");
      if (new_page) pg3 = checked(table_row ? pg_raw : ce.b * a.cache.max_pages + lk_p_prev);
      if (!lookup) pg3 = -1;
    }
    GQLA_STAMP(3);
  };
  using T_ = std::true_type;
  using F_ = std::false_type;
  iteration(0, T_{}, F_{}, F_{});
  {
    int it = 1;
#pragma unroll 1
    for (; it + 2 < n_tiles; ++it) iteration(it, T_{}, T_{}, T_{});
#pragma unroll 1
    for (; it < n_tiles; ++it) iteration(it, T_{}, T_{}, F_{});
  }
  iteration(n_tiles, F_{}, T_{}, F_{});

#ifdef GQLA_PHASE_TIMING
  if (threadIdx.x == 0) {
    for (int k = 0; k < 8; ++k) atomicAdd(&gqla_phase_cycles[k], (unsigned long long)ph_[k]);
    atomicAdd(&gqla_phase_cycles[15], (unsigned long long)n_tiles);
    atomicAdd(&gqla_phase_cycles[14], (unsigned long long)(__builtin_readcyclecounter() - t_entry_));
    atomicAdd(&gqla_phase_cycles[13], 1ull);
  }
#endif
  // ---- chunk partial: O^T / l as bf16 in latent space, log-sum-exp per row ----
  const float l_tot = pair_sum(l_run);
  __syncthreads();  // every wave is done with the exchange
  float* inv_l = (float*)(smem + EX);
  if (h == 0) inv_l[wave * 32 + n] = l_tot > 0.f ? 1.f / l_tot : 0.f;
  __builtin_amdgcn_s_waitcnt(0xc07f);
  __syncthreads();
  if (h == 0)
    a.part_lse[(int64_t)chunk * a.M + rho] = l_tot > 0.f ? (m_ref + fast_log2(l_tot)) * kLn2 : GQLA_NEG_INF;
#pragma unroll
  for (int rb = 0; rb < 4; ++rb) {
    const int row = row0 + rb * 32 + n;
    const float inv = inv_l[rb * 32 + n];
    // dims 4 h .. 4 h + 3 of vector 16 wave + 4 d + q of the lane's row: 512 contiguous bytes per store instruction
    __bf16* po = (__bf16*)a.part_o + part_vec_index(chunk, row, a.M, RKV / 8, 16 * wave) * 8 + 4 * h;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      float x[16];
      acc_read(4 * d + rb, rb == 0 && d == 0, x);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        u32x2 v = {pack_bf16(x[4 * q] * inv, x[4 * q + 1] * inv), pack_bf16(x[4 * q + 2] * inv, x[4 * q + 3] * inv)};
        *(u32x2*)(po + (4 * d + q) * (32 * 8)) = v;
      }
    }
  }
}

// ---- MQA-absorb decode over an 8-bit latent cache (c_kv as E4M3 codes with one scale, k_R in 16 bits) ----
// The paper names quantised caches as complementary and fixes no format (Sec. 2; Sec. 5.1, item (i)); the page format is
// this library's (gqla.h): code rows [P][r_kv] back to back, then k_R [P][d_r] in 16 bits -- r_kv + 2 d_r bytes per token.
// The decode is the MQA-absorb equation on c' = value(code) * scale.  Same mapping of rows to waves as
// decode_absorb_bf16_kernel above (one wave per 32 rows, or four waves sharing 32 rows), same MFMAs: the codes are
// widened to bf16 ONCE per tile on their way into LDS, by the wave that fetched them, so that every row block reads
// ready-made bf16 fragments:
//   tile it+2:  four 16-byte loads of codes per lane (whole 128-byte lines: 8 rows x 128 code bytes per wave
//               instruction) and one of k_R, in flight in 20 registers for one whole iteration
//   tile it+1:  its codes (requested one iteration ago) are widened (v_cvt_scalef32_pk_bf16_fp8, exact) and written to
//               the idle one of two LDS tile buffers in the panel layout of gqla_lds.h -- the lanes of a 16-lane group
//               cover 4 rows x 4 chunk pairs, which the layout's XOR spreads over all 64 banks; its k_R rows (already
//               16-bit) are written as they came
// Everything in flight is an ordinary load into registers: the compiler places every wait itself, and no wait of this
// kernel is counted by hand.
// The scale enters twice, both times outside the MFMAs: on the content part of the logits (between the latent k-steps
// and the RoPE k-steps of S^T) and on the normalised output.
__device__ __forceinline__ bf16x8 widen_e4m3x8(uint32_t w0, uint32_t w1) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2v;
  const bf16x2v p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, false), p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, true);
  const bf16x2v p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, false), p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, true);
  const u32x4 r = {__builtin_bit_cast(uint32_t, p0), __builtin_bit_cast(uint32_t, p1), __builtin_bit_cast(uint32_t, p2), __builtin_bit_cast(uint32_t, p3)};
  return __builtin_bit_cast(bf16x8, r);
}

template <int RKV, int DR, int SPLIT>
__global__ void __launch_bounds__(256) decode_absorb_fp8_kernel(DecodeArgs a, int row_blocks, float c_scale) {
  constexpr int W = RKV + DR;        // elements per latent row (in LDS: all bf16)
  constexpr int NP = W / 64;         // 128-byte panels per latent row in LDS
  constexpr int PANEL = kTile * 128; // bytes per panel
  constexpr int KS = W / 16;         // k-steps of the key contraction
  constexpr int KS_C = RKV / 16;     // ... of which over the latent (the rest over the RoPE key)
  constexpr int DT = RKV / 32;       // 32-wide tiles of the latent output
  constexpr int TILE_BYTES = kTile * W * 2;
  constexpr int RPB = kRowsPerBlock / SPLIT;
  constexpr int KB = 4 / SPLIT;
  constexpr int DTW = DT / SPLIT;
  static_assert(SPLIT == 1 || SPLIT == 4, "one wave or the whole workgroup per 32 rows");
  static_assert(RKV == 512 && DR == 64, "the staging below is written for 8 code panels of 64 bytes per row and one k_R panel");
  static_assert(DT == 16, "O^T fills the 256 accumulation registers exactly");
  extern __shared__ __attribute__((aligned(16))) char smem[];

  int chunk, rbk;
  {
    const int id = blockIdx.x;
    const int grp = id / (8 * row_blocks), rem = id % (8 * row_blocks);
    rbk = rem / 8;
    chunk = grp * 8 + rem % 8;
  }
  if (chunk >= a.n_chunks) return;  // whole workgroup leaves together
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 31, h = lane >> 5;
  const ChunkEntry ce = a.chunks[chunk];

  const int part = wave & (SPLIT - 1), team = wave / SPLIT;
  const int rho = rbk * RPB + team * 32 + n;  // row = t * h_q + i
  const bool row_ok = rho < a.M;
  const int t = row_ok ? rho / a.h_q : 0;
  const int vis_end = row_ok ? min(ce.tok_end, ce.L - a.s_q + t + 1) : 0;
  const int unmasked_end = min(ce.tok_end, ce.L - a.s_q + 1);
  const bool wave_active = SPLIT > 1 || rbk * RPB + team * 32 < a.M;

  const int P = a.cache.page_size;
  const char* pool = (const char*)a.cache.pool;
  const int64_t page_bytes = (int64_t)P * (RKV + 2 * DR);
  const int32_t* table_row = a.cache.page_table ? a.cache.page_table + (int64_t)ce.b * a.cache.max_pages : nullptr;
  auto checked = [&](int32_t pg) -> int32_t { return ((uint32_t)pg < (uint32_t)a.cache.num_pages) ? pg : -1; };
  // first code row / first k_R row of a tile: page pg (page 0 for an id outside the pool; such a tile is zeroed), slot `slot`
  auto code_src = [&](int32_t pg, int slot) -> const char* { return pool + (int64_t)(pg >= 0 ? pg : 0) * page_bytes + (int64_t)slot * RKV; };
  auto kr_src = [&](int32_t pg, int slot) -> const char* {
    return pool + (int64_t)(pg >= 0 ? pg : 0) * page_bytes + (int64_t)P * RKV + (int64_t)slot * (DR * 2);
  };

  uint32_t kbase[KB], vbase;
  {
#pragma unroll
    for (int b = 0; b < KB; ++b) kbase[b] = n * 128 + (((2 * (part * KB + b) + h) ^ lds_swz(n)) << 4);
    const int i16 = lane & 15, e = i16 >> 2, q = i16 & 3, g1 = (lane >> 4) & 1;
    vbase = (4 * h + e) * 128 + (((2 * g1 + (q >> 1)) ^ (2 * h + (e >> 1))) << 4) + (q & 1) * 8;
    vbase += part * (DTW / 2) * PANEL;
  }
  // staging: load i (0..3) of this lane fetches the 16 codes of row R, dims 16*k .. 16*k+15, k = 4*(2i + hp) + kq, and
  // writes them as chunks 2k, 2k+1 of row R: panel 2i + hp, in-panel slots (2kq) ^ swz, (2kq+1) ^ swz
  const int st_R = 8 * wave + 4 * ((lane >> 4) & 1) + ((lane >> 2) & 3), st_kq = lane & 3, st_hp = lane >> 5;
  const uint32_t st_goff = st_R * RKV + (4 * st_hp + st_kq) * 16;
  const uint32_t st_w0 = st_R * 128 + (((2 * st_kq) ^ lds_swz(st_R)) << 4) + st_hp * PANEL;
  const uint32_t st_w1 = st_R * 128 + (((2 * st_kq + 1) ^ lds_swz(st_R)) << 4) + st_hp * PANEL;
  // ... and one 16-byte piece of k_R: row kr_R, chunk lane % 8 (eight lanes per 128-byte row)
  const int kr_R = 8 * wave + (lane >> 3);
  const uint32_t kr_goff = kr_R * (DR * 2) + (lane & 7) * 16;
  const uint32_t kr_w = (RKV / 64) * PANEL + kr_R * 128 + (((lane & 7) ^ lds_swz(kr_R)) << 4);

  acc_zero();
  float m_ref = GQLA_NEG_INF, l_run = 0.f;
  const int n_tiles = (ce.tok_end - ce.tok_begin + kTile - 1) / kTile;

  u32x4 codes[4], kr16;  // in flight: 4 x 16 codes and 8 elements of k_R per lane
  auto load_tile = [&](int32_t pg, int slot) __attribute__((always_inline)) {
    const char* src = code_src(pg, slot);
#pragma unroll
    for (int i = 0; i < 4; ++i) codes[i] = __builtin_nontemporal_load((const u32x4*)(src + st_goff + i * 128));
    kr16 = __builtin_nontemporal_load((const u32x4*)(kr_src(pg, slot) + kr_goff));
  };
  // widen the codes in flight and write them as rows of the bf16 tile at `slot`; rows >= valid are written as zeros
  // (slots past the chunk end hold whatever the page holds, and 0 * v must stay 0)
  auto write_tile = [&](char* slot, int valid) __attribute__((always_inline)) {
    const bool keep = st_R < valid;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      u32x4 lo = __builtin_bit_cast(u32x4, widen_e4m3x8(codes[i][0], codes[i][1]));
      u32x4 hi = __builtin_bit_cast(u32x4, widen_e4m3x8(codes[i][2], codes[i][3]));
      if (!keep) lo = hi = u32x4{0u, 0u, 0u, 0u};
      *(u32x4*)(slot + st_w0 + i * 2 * PANEL) = lo;
      *(u32x4*)(slot + st_w1 + i * 2 * PANEL) = hi;
    }
    *(u32x4*)(slot + kr_w) = kr_R < valid ? kr16 : u32x4{0u, 0u, 0u, 0u};
  };
  auto page_now = [&](int tile) -> int32_t {  // synchronous lookup (start-up only)
    const int p = (ce.tok_begin + tile * kTile) / P;
    return checked(table_row ? table_row[p] : ce.b * a.cache.max_pages + p);
  };

  // queries of this lane's row, as B fragments (requested first: their latency overlaps the first tile's)
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
  // start-up: tile 0 into buffer 0, codes of tile 1 in flight
  int32_t pg_cur = page_now(0);
  int32_t pg_n1 = n_tiles > 1 ? page_now(1) : -1;  // page of tile it+1
  load_tile(pg_cur, 0);
  // the query loads complete here
#pragma unroll
  for (int k = 0; k < KS / SPLIT; k += 9)
    asm volatile("" : "+v"(qf[k]), "+v"(qf[k + 1]), "+v"(qf[k + 2]), "+v"(qf[k + 3]), "+v"(qf[k + 4]), "+v"(qf[k + 5]),
                      "+v"(qf[k + 6]), "+v"(qf[k + 7]), "+v"(qf[k + 8]));
  static_assert((KS / SPLIT) % 9 == 0, "query fragments are touched nine at a time");
  write_tile(smem, pg_cur >= 0 ? min(kTile, ce.tok_end - ce.tok_begin) : 0);
  if (n_tiles > 1) load_tile(pg_n1, kTile % P);
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the tile is written
  __syncthreads();
  int32_t pg_lane = 0;
  int lane_zero;
  asm volatile("v_mov_b32 %0, 0" : "=v"(lane_zero));

#pragma unroll 1
  for (int it = 0; it < n_tiles; ++it) {
    const int tok = ce.tok_begin + it * kTile;
    const char* buf = smem + (it & 1) * TILE_BYTES;
    char* nbuf = smem + ((it + 1) & 1) * TILE_BYTES;
    // page of tile it+2: looked up when that tile starts a page, consumed behind the S phase.  An ordinary load into a
    // vector register (every lane reads the same entry; the lane-dependent zero keeps the compiler from turning it into
    // a load-and-wait on the spot), so that the compiler itself waits for it where the value is first read.  (A scalar
    // load issued and awaited by hand is not safe here: this loop's control flow makes the compiler copy the value
    // between registers, and a copy ahead of the hand-placed wait reads the register while the load is pending.)
    const int tok2 = tok + 2 * kTile;
    const bool has2 = it + 2 < n_tiles;
    const bool new_page = has2 && (tok2 % P) == 0;
    if (new_page && table_row) pg_lane = table_row[tok2 / P + lane_zero];
    const bool tile_ok = pg_cur >= 0;

    // tile it+1 into the idle buffer (every wave passed the last barrier: nobody reads tile it-1 any more), the codes of
    // tile it+2 into flight.  No LDS read of this wave is outstanding where this is called.
    auto stage_step = [&]() __attribute__((always_inline)) {
      const int32_t pg_n2 = !has2 ? -1 : (new_page ? checked(table_row ? __builtin_amdgcn_readfirstlane(pg_lane)
                                                                           : ce.b * a.cache.max_pages + tok2 / P) : pg_n1);
      if (it + 1 < n_tiles) {
        write_tile(nbuf, pg_n1 >= 0 ? min(kTile, ce.tok_end - (tok + kTile)) : 0);
      }
      if (has2) load_tile(pg_n2, tok2 % P);
      pg_cur = pg_n1;  // (used again only in the next iteration)
      pg_n1 = pg_n2;
    };
    auto end_of_tile = [&]() __attribute__((always_inline)) {
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's rows of tile it+1 are written
      __syncthreads();
    };
    const bool need_mask = (tok + kTile > unmasked_end) || !row_ok || !tile_ok;
    const int lim = tile_ok ? vis_end : 0;

    // ---- S^T[token][row] = Kt * Qhat^T: latent k-steps, the scale, RoPE k-steps ----
    // (waves without query rows only stage: ONE call site of stage_step for both kinds, so that the codes in flight
    // live in the same registers on every path and nothing has to wait for them before the staging itself)
    f32x16 s;
    if (wave_active) {
      bf16x8 f[2][KB];  // fragment batches: loads run one batch (one panel) ahead of their use
#pragma unroll
      for (int b = 0; b < KB; ++b) f[0][b] = *(const bf16x8*)(buf + kbase[b]);
#pragma unroll
      for (int a4 = 0; a4 < KS / 4; ++a4) {
        if (a4 + 1 < KS / 4) {
#pragma unroll
          for (int b = 0; b < KB; ++b) f[(a4 + 1) & 1][b] = *(const bf16x8*)(buf + kbase[b] + ((a4 + 1) * PANEL));
        }
        __builtin_amdgcn_sched_barrier(0);
        if (a4 == KS_C / 4) {  // the latent part is complete: the cache's scale, before the RoPE part is added
          asm volatile("s_nop 15\n\ts_nop 7" : "+v"(s));
#pragma unroll
          for (int i = 0; i < 16; ++i) s[i] *= c_scale;
          asm volatile("s_nop 1" : "+v"(s));
        }
#pragma unroll
        for (int b = 0; b < KB; ++b) {
          if (a4 == 0 && b == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(s) : "v"(f[0][0]), "v"(qf[0]));
          else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(f[a4 & 1][b]), "v"(qf[a4 * KB + b]));
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    stage_step();
    if (wave_active) {
    // first batch of value fragments: issued now, consumed after the softmax
    i16x4 r[2][4][2];
    auto load_v = [&](int slot, int u, int p4) __attribute__((always_inline)) {
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const int dt = 4 * p4 + d;
        const int off = (dt >> 1) * PANEL + (16 * u) * 128;
        r[slot][d][0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(buf + vbase + (off + 64 * (dt & 1))));
        r[slot][d][1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(buf + vbase + (off + 8 * 128 + 64 * (1 - (dt & 1)))));
      }
    };
    constexpr int NBT = 2 * (DTW / 4);
    asm volatile("s_nop 15\n\ts_nop 7" : "+v"(s));  // the matrix pipeline's result is not interlocked against vector-ALU reads
    if constexpr (SPLIT > 1) {
      // team sum of the partial S^T: [wave][quarter][lane] 16-byte slots behind the two tile buffers.  (The scale was
      // applied to every wave's latent part; the RoPE part is spread over the waves like the latent part.)
      char* ex = smem + 2 * TILE_BYTES;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *(f32x4*)(ex + wave * 4096 + q * 1024 + lane * 16) = f32x4{s[4 * q], s[4 * q + 1], s[4 * q + 2], s[4 * q + 3]};
      __builtin_amdgcn_s_waitcnt(0xc07f);
      __syncthreads();  // the next write to these slots comes after the end-of-tile barrier, which follows these reads
#pragma unroll
      for (int w = 0; w < SPLIT; ++w)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 x = *(const f32x4*)(ex + (team * SPLIT + w) * 4096 + q * 1024 + lane * 16);
#pragma unroll
          for (int e = 0; e < 4; ++e) s[4 * q + e] = (w == 0) ? x[e] : s[4 * q + e] + x[e];
        }
    }
    load_v(0, 0, 0);

    // ---- online softmax (base 2); register i is token tok + 8*(i/4) + 4*h + i%4 ----
    if (__builtin_amdgcn_ballot_w64(need_mask) != 0) {
      int dist = lim - tok - 4 * h;
      asm volatile("" : "+v"(dist));
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (need_mask && 8 * (i >> 2) + (i & 3) >= dist) s[i] = GQLA_NEG_INF;
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
    bf16x8 pf[2];
    {
      float p[16], psum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        p[e] = fast_exp2(__builtin_fmaf(s[e], a.scale_log2e, -m_use));
        psum += p[e];
      }
      l_run += psum;
      const u32x4 w0 = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
      const u32x4 w1 = {pack_bf16(p[8], p[9]), pack_bf16(p[10], p[11]), pack_bf16(p[12], p[13]), pack_bf16(p[14], p[15])};
      pf[0] = __builtin_bit_cast(bf16x8, w0);
      pf[1] = __builtin_bit_cast(bf16x8, w1);
    }
    asm volatile("s_nop 1" : "+v"(pf[0]), "+v"(pf[1]));  // two wait states between a vector-ALU write and an MFMA that reads it
    __builtin_amdgcn_sched_barrier(0);

    // ---- O^T[r][row] += C^T * P^T, value fragments one batch of four tiles ahead ----
#pragma unroll
    for (int bt = 0; bt < NBT; ++bt) {
      const int u = bt / (DTW / 4), p4 = bt % (DTW / 4);
      if (bt + 1 < NBT) load_v((bt + 1) & 1, (bt + 1) / (DTW / 4), (bt + 1) % (DTW / 4));
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const i16x4 lo = r[bt & 1][d][0], hi = r[bt & 1][d][1];
        const i16x8 fr = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        acc_mfma(4 * p4 + d, __builtin_bit_cast(bf16x8, fr), pf[u]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    }
    end_of_tile();
  }

  const float l_tot = pair_sum(l_run);
  if (!row_ok) return;
  const float inv = (l_tot > 0.f ? 1.f / l_tot : 0.f) * c_scale;  // o_hat = scale * sum_s p_s value(code_s)
  const int64_t prow = (int64_t)chunk * a.M + rho;
  // this lane holds dims 4 h .. 4 h + 3 of vector 4 (part DTW + dt) + q of its row: with consecutive rows in consecutive
  // lanes a store instruction writes 512 contiguous bytes
  __bf16* po = (__bf16*)a.part_o + part_vec_index(chunk, rho, a.M, RKV / 8, 0) * 8 + 4 * h;
#pragma unroll
  for (int dt = 0; dt < DTW; ++dt) {
    float x[16];
    acc_read(dt, dt == 0, x);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      u32x2 v = {pack_bf16(x[4 * q] * inv, x[4 * q + 1] * inv), pack_bf16(x[4 * q + 2] * inv, x[4 * q + 3] * inv)};
      *(u32x2*)(po + ((part * DTW + dt) * 4 + q) * (32 * 8)) = v;
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
  // vector 2 (KSW wave + ksl) + h of the lane's row, chunk 0 (see part_vec_index: consecutive rows are 16 bytes apart)
  const __bf16* po = (const __bf16*)a.part_o + part_vec_index(0, rho, a.M, RKV / 8, 2 * KSW * wave + h) * 8;
  const int64_t chunk_stride = (int64_t)((a.M + 31) / 32) * 32 * RKV;   // elements from one chunk's partials to the next
  for (int sb = s0; sb < s1; sb += kNB) {
    float l[kNB];
    u32x4 v[kNB][KSW];
#pragma unroll
    for (int k = 0; k < kNB; ++k) {
      const int sc = min(sb + k, s1 - 1);  // clamped: a chunk beyond the range is loaded again and given weight 0
      l[k] = a.part_lse[(int64_t)sc * a.M + rho];
#pragma unroll
      for (int ksl = 0; ksl < KSW; ++ksl) v[k][ksl] = *(const u32x4*)(po + sc * chunk_stride + ksl * (2 * 32 * 8));
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

static hipError_t launch_decode_absorb_shared(const DecodeArgs& a, hipStream_t s) {
  constexpr int kLds = kSlots * kTile * (512 + 64) * 2 + 2 * 8192;  // tile ring + the double-buffered exchange: all 160 KB
  static const hipError_t attr =
      hipFuncSetAttribute((const void*)decode_absorb_shared_bf16_kernel<512, 64>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
  if (attr != hipSuccess) return attr;
  const int row_blocks = a.M / kRowsPerBlock;
  const int chunks_padded = (a.n_chunks + 7) / 8 * 8;
  decode_absorb_shared_bf16_kernel<512, 64><<<chunks_padded * row_blocks, 256, kLds, s>>>(a, row_blocks);
  return hipGetLastError();
}

hipError_t launch_decode_absorb_bf16(const DecodeArgs& a, hipStream_t s) {
  // At most 32 query rows: the four waves share them, so that none is left without work.  More rows but few chunks
  // (small batches): one workgroup per (chunk, 32 rows) with the four waves sharing its rows, as long as all of them
  // still run at once -- four times the workgroups, each with a shorter tile (the tiles' re-reads hit the L2, and
  // with so few chunks the chip is nowhere near its memory rate).
  const int chunks_padded = (a.n_chunks + 7) / 8 * 8;
  if (a.M <= 32 || chunks_padded * ((a.M + 31) / 32) <= a.num_cus) return launch_decode_absorb_split<4>(a, s);
  // whole blocks of 128 rows (h_q s_q a multiple of 128): the pipelined kernel with shared probabilities; other row
  // counts above 32: one wave per 32 rows, each with its own probabilities
  return a.M % kRowsPerBlock == 0 ? launch_decode_absorb_shared(a, s) : launch_decode_absorb_split<1>(a, s);
}

template <int SPLIT>
static hipError_t launch_decode_absorb_fp8_split(const DecodeArgs& a, float c_scale, hipStream_t s) {
  constexpr int kLds = 2 * kTile * (512 + 64) * 2 + (SPLIT > 1 ? 4 * 4096 : 0);  // two bf16 tile buffers (+ the team exchange)
  static const hipError_t attr =
      hipFuncSetAttribute((const void*)decode_absorb_fp8_kernel<512, 64, SPLIT>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
  if (attr != hipSuccess) return attr;
  const int row_blocks = (a.M + kRowsPerBlock / SPLIT - 1) / (kRowsPerBlock / SPLIT);
  const int chunks_padded = (a.n_chunks + 7) / 8 * 8;
  decode_absorb_fp8_kernel<512, 64, SPLIT><<<chunks_padded * row_blocks, 256, kLds, s>>>(a, row_blocks, c_scale);
  return hipGetLastError();
}

hipError_t launch_decode_absorb_fp8(const DecodeArgs& a, float c_scale, hipStream_t s) {
  // the same choice of row mapping as for the 16-bit cache
  const int chunks_padded = (a.n_chunks + 7) / 8 * 8;
  if (a.M <= 32 || chunks_padded * ((a.M + 31) / 32) <= a.num_cus) return launch_decode_absorb_fp8_split<4>(a, c_scale, s);
  return launch_decode_absorb_fp8_split<1>(a, c_scale, s);
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
