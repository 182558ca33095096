// Similarity + matching stage of Chunked Soft Matching (Sec. 5.2, Eq. 2) for gfx950.
//
// Per chunk of L tokens: A = tokens at even offsets (sources), B = odd offsets (destinations).
// For every A token i:  j*(i) = argmax_j  k_i.k_j / (|k_i||k_j|)  (lowest j on ties) and that
// maximum.  The |A| x |B| similarity matrix lives only in MFMA accumulators.
//
// Three bf16 kernels.  Common to all: 64 A rows per wave held as MFMA operands in registers; the
// MFMA computes S^T (B index on the M side) so that a lane's 16 accumulators of a 32x32 tile all
// belong to ONE A row (no cross-lane step until the very end); inverse norms come from the same
// bytes (v_dot2 on the packed pairs): the B rows' while they are staged into LDS, the A rows'
// from the operand registers.
//   match_bf16_kernel: one workgroup = (sequence, chunk, block of A rows); 8 waves (512 A rows) for
// chunks above 512 tokens, 4 waves otherwise.  The A rows are staged once through LDS; the chunk's
// B rows stream through two LDS panels of 128 rows (global -> registers -> LDS, one barrier per
// panel).  Blocks made of full tiles fold tile q into the running maxima while the MFMAs of tile
// q+1 run; ragged blocks take the maximum first and resolve the index only for tiles that raise
// some lane's maximum.
//   match_small_bf16_kernel (whole chunks of 64, 128 or 256 tokens): several chunks per workgroup, see below.
//   match_stream_bf16_kernel (dim 128, whole chunks of 1024 or 2048 tokens): persistent, see below.
#include <type_traits>
#include <utility>

#include "ckv_internal.h"
#include "ckv_device.h"

namespace ckv {
namespace {

template <class F, int... S>
__device__ __forceinline__ void static_for(F&& f, std::integer_sequence<int, S...>) {
  (f(std::integral_constant<int, S>{}), ...);
}

constexpr int kThreads = 256;
constexpr int kRowsPerWave = 64;                 // two 32-row MFMA tiles
constexpr int kPanel = 128;                      // B rows per LDS panel

// NW waves x 64 A rows per workgroup: 4 waves (two workgroups per CU) for chunks of up to 512 tokens,
// 8 waves (one workgroup per CU) for larger chunks, so that the B rows of a 1024-token chunk are
// fetched, normed and written to LDS once instead of once per 256 A rows.
// PAGED: K is a block pool and the rows are reached through a block table (see PagedSide); the pool
// rows of the chunk's blocks are staged in LDS first.
template <int D, int NW, bool PAGED>
__global__ __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) void match_bf16_kernel(
    const __bf16* __restrict__ K, TensorView kv, int seq, int chunk, int n_chunks, int g_first, int a_blocks,
    int total_work, int per_xcd, int32_t* __restrict__ dst_local, float* __restrict__ score, PagedSide paged) {
  constexpr int OCT = D / 8;                       // 16-byte pieces per key row
  constexpr int ROWB = D * 2;                      // bytes per row
  constexpr int KEYSHIFT = (ROWB == 256) ? 0 : 1;  // rows per 256 B of LDS = 1 << KEYSHIFT
  constexpr int KSTEPS = D / 16;
  constexpr int THREADS = NW * 64;
  constexpr int ABLOCK = NW * kRowsPerWave;        // A rows per workgroup
  constexpr int PANELS_B = (ABLOCK > 2 * kPanel ? ABLOCK : 2 * kPanel) * ROWB;   // staging area: A block or 2 panels
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* panel0 = smem;                                // 2 panels of kPanel rows; the A
  float* invb = reinterpret_cast<float*>(smem + PANELS_B);           // block is staged over them
  int32_t* s_rb = reinterpret_cast<int32_t*>(invb + 2 * kPanel);     // PAGED: pool rows of the chunk's blocks

  const int w = xcd_remap(blockIdx.x, per_xcd);
  if (w >= total_work) return;
  const int ab = w % a_blocks;
  const int g = g_first + (w / a_blocks) % n_chunks;     // the launch covers chunks g_first .. g_first + n_chunks - 1
  const int bh = w / (a_blocks * n_chunks);
  const int g0 = g * chunk;
  const int L = min(chunk, seq - g0);
  const int nA = (L + 1) >> 1, nB = L >> 1;
  const int a0 = ab * ABLOCK;
  if (a0 >= nA) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_src = n_sources(seq, chunk);
  const int64_t out_base = (int64_t)bh * n_src + (int64_t)g * (chunk >> 1);
  if (nB == 0) {  // a one-token tail chunk: nothing to match
    if (tid == 0) { dst_local[out_base] = -1; score[out_base] = 0.f; }
    return;
  }
  const __bf16* Kseq = PAGED ? K : K + kv.seq_base(bh) + (int64_t)g0 * kv.stride_s;
  RowBases rows{};
  const int u0 = paged.tok0 + g0;              // PAGED: the chunk's first token within its sequence
  if (PAGED) {
    rows = stage_row_bases(s_rb, paged, bh / kv.heads, bh % kv.heads, kv.heads, u0, u0 + L - 1, tid, NW * 64);
    __syncthreads();
  }
  // address of token u of the chunk (the 16-byte piece of this thread is added by the caller)
  auto tok_ptr = [&](int u) -> const __bf16* {
    if (PAGED) return K + (int64_t)rows.row(u0 + u) * D;
    return Kseq + (int64_t)u * kv.stride_s;
  };

  auto swz = [](int row, int piece) -> int {
    return row * ROWB + (((piece ^ (row >> KEYSHIFT)) & (OCT - 1)) << 4);
  };

  // ---- stage the A block (even offsets) and its inverse norms --------------------------------
  // All global loads are issued before the first use (rows past the end re-read the last valid
  // row and are zeroed), together with the first B panel, so one memory latency covers both.
  constexpr int PIECES = kPanel * OCT / THREADS;   // 16-byte pieces per thread per panel
  Piece stage[PIECES];
  const int piece = tid % OCT, r0 = tid / OCT;
  constexpr int ROWS_PER_PASS = THREADS / OCT;
  // every thread walks its own column of 16-byte pieces: row r0 + it*ROWS_PER_PASS of a panel
  const __bf16* Bcol = Kseq + kv.stride_s + piece * 8;          // B row j lives at token 2j+1
  const int64_t row_pitch = 2 * kv.stride_s;
  auto load_panel = [&](int pbase) {
    if (pbase + kPanel > nB) {   // ragged last panel (uniform branch): clamp to the last row
#pragma unroll
      for (int it = 0; it < PIECES; ++it) {
        const int j = min(pbase + r0 + it * ROWS_PER_PASS, nB - 1);
        stage[it].u = PAGED ? *reinterpret_cast<const uint4*>(tok_ptr(2 * j + 1) + piece * 8)
                            : *reinterpret_cast<const uint4*>(Bcol + j * row_pitch);
      }
    } else if (PAGED) {
#pragma unroll
      for (int it = 0; it < PIECES; ++it)
        stage[it].u = *reinterpret_cast<const uint4*>(tok_ptr(2 * (pbase + r0 + it * ROWS_PER_PASS) + 1) + piece * 8);
    } else {
      const __bf16* src = Bcol + (int64_t)(pbase + r0) * row_pitch;
#pragma unroll
      for (int it = 0; it < PIECES; ++it)
        stage[it].u = *reinterpret_cast<const uint4*>(src + it * ROWS_PER_PASS * row_pitch);
    }
  };
  // ROWS_PER_PASS is a multiple of the swizzle period, so a thread's pieces sit at a fixed
  // offset plus a multiple of ROWS_PER_PASS rows
  static_assert(ROWS_PER_PASS % (OCT << KEYSHIFT) == 0, "swizzle period");
  const int lds_piece0 = swz(r0, piece);
  auto store_panel = [&](int buf, int pbase) {
    unsigned char* pb = panel0 + buf * kPanel * ROWB + lds_piece0;
    if (pbase + kPanel > nB) {   // ragged last panel (uniform branch): rows past the end are zero
#pragma unroll
      for (int it = 0; it < PIECES; ++it)
        if (pbase + r0 + it * ROWS_PER_PASS >= nB) stage[it].u = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int it = 0; it < PIECES; ++it) {
      const float ss = row_sum<OCT>(sumsq8(stage[it]));
      *reinterpret_cast<uint4*>(pb + it * ROWS_PER_PASS * ROWB) = stage[it].u;
      if (piece == 0) invb[buf * kPanel + r0 + it * ROWS_PER_PASS] = inv_norm(ss);
    }
  };
  // panels are visited starting at the one that holds this block's own neighbourhood (keys are
  // most similar to their neighbours, so the running maxima settle in the first panel)
  const int n_panels = div_up(nB, kPanel);
  // a block of full tiles takes the software-pipelined loop below, panels in increasing order
  const bool pipelined = (NW == 8) && (a0 + ABLOCK <= nA) && (nB % kPanel == 0);
  const int p_first = pipelined ? 0 : min(a0 / kPanel, n_panels - 1);
  {
    constexpr int APIECES = ABLOCK * OCT / THREADS;
    Piece xa[APIECES];
#pragma unroll
    for (int it = 0; it < APIECES; ++it) {
      const int a = min(a0 + r0 + it * ROWS_PER_PASS, nA - 1);
      xa[it].u = *reinterpret_cast<const uint4*>(tok_ptr(2 * a) + piece * 8);
    }
    load_panel(p_first * kPanel);
    if (a0 + ABLOCK > nA) {
#pragma unroll
      for (int it = 0; it < APIECES; ++it)
        if (a0 + r0 + it * ROWS_PER_PASS >= nA) xa[it].u = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int it = 0; it < APIECES; ++it)
      *reinterpret_cast<uint4*>(panel0 + lds_piece0 + it * ROWS_PER_PASS * ROWB) = xa[it].u;
  }
  __syncthreads();
  bf16x8 afrag[2][KSTEPS];
  const int half = lane >> 5, col = lane & 31;
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    const int row = wave * kRowsPerWave + rt * 32 + col;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s)
      afrag[rt][s] = *reinterpret_cast<const bf16x8*>(panel0 + swz(row, 2 * s + half));
  }
  // 1/|k_i| of this lane's two A rows, from the operand registers
  const float my_inva[2] = {inv_norm_of_operand_row<KSTEPS>(afrag[0]), inv_norm_of_operand_row<KSTEPS>(afrag[1])};
  __syncthreads();

  // ---- stream B panels -----------------------------------------------------------------------
  float best[2] = {-INFINITY, -INFINITY};
  int bestj[2] = {0, 0};
  const bool wave_active = (a0 + wave * kRowsPerWave) < nA;
  // LDS byte offsets of this lane's B fragments inside a 32-row tile: the swizzle key of row
  // ct*32 + col only depends on col, so tile and buffer offsets are compile-time immediates
  int boff[KSTEPS];
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) boff[s] = swz(col, 2 * s + half);
  const float* ib_lane = invb + 4 * half;
  auto compute_tiles = [&](auto buf_c, auto full_c, int pbase, int rows_here) {
    constexpr int BUF = decltype(buf_c)::value;
    constexpr bool FULL = decltype(full_c)::value;
    const unsigned char* pb = panel0 + BUF * kPanel * ROWB;
    const int n_ct = FULL ? kPanel / 32 : div_up(rows_here, 32);
#pragma unroll
    for (int ct = 0; ct < kPanel / 32; ++ct) {
      if (!FULL && ct >= n_ct) break;
      f32x16 acc0 = {0}, acc1 = {0};
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s) {
        const bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(pb + ct * 32 * ROWB + boff[s]);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag, afrag[0][s], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag, afrag[1][s], acc1, 0, 0, 0);
      }
      // accumulator r of this lane: B row 8*(r/4) + 4*half + r%4 of the tile, A row = col
      f32x4 ib[4];
#pragma unroll
      for (int qd = 0; qd < 4; ++qd)
        ib[qd] = *reinterpret_cast<const f32x4*>(ib_lane + BUF * kPanel + ct * 32 + 8 * qd);
      const int jbase = pbase + ct * 32;
      const int valid = rows_here - ct * 32;      // rows of this tile that exist (>= 32: all)
      if (FULL || valid >= 32) {
        tile_argmax<false>(acc0, ib, jbase, half, valid, best[0], bestj[0]);
        tile_argmax<false>(acc1, ib, jbase, half, valid, best[1], bestj[1]);
      } else {
        tile_argmax<true>(acc0, ib, jbase, half, valid, best[0], bestj[0]);
        tile_argmax<true>(acc1, ib, jbase, half, valid, best[1], bestj[1]);
      }
    }
  };
  if (NW == 8 && pipelined) {
    // A stage issues the MFMAs of one tile and, one slice of vector work behind each of them,
    // folds the PREVIOUS tile's accumulators into the running maxima: matrix pipe and vector
    // ALU of the wave work side by side instead of taking turns.  B fragments are read from
    // LDS two k-steps ahead.
    const int jl = 4 * half;
    auto load_ib = [&](auto row_c, f32x4 (&ib)[4]) {
#pragma unroll
      for (int qd = 0; qd < 4; ++qd)
        ib[qd] = *reinterpret_cast<const f32x4*>(ib_lane + decltype(row_c)::value + 8 * qd);
    };
    auto stage = [&](auto row_c, auto fold_c, f32x16& n0, f32x16& n1, f32x16& c0, f32x16& c1,
                     const f32x4 (&ib)[4], f32x4 (&ib_next)[4], int jlane) {
      constexpr int ROW = decltype(row_c)::value;      // first row of the B tile in the LDS panels
      constexpr bool FOLD = decltype(fold_c)::value;
      constexpr int SPS = (kFoldSteps + 2 * KSTEPS - 1) / (2 * KSTEPS);   // fold steps per slice
      const unsigned char* pb = panel0 + ROW * ROWB;
      bf16x8 bq[KSTEPS];
      bq[0] = *reinterpret_cast<const bf16x8*>(pb + boff[0]);
      bq[1] = *reinterpret_cast<const bf16x8*>(pb + boff[1]);
      FoldRegs f;
      auto kstep = [&](auto s_c) {
        constexpr int S = decltype(s_c)::value;
        if constexpr (S + 2 < KSTEPS) bq[S + 2] = *reinterpret_cast<const bf16x8*>(pb + boff[S + 2]);
        n0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq[S], afrag[0][S], S == 0 ? f32x16{0} : n0, 0, 0, 0);
        if constexpr (FOLD) fold_steps<2 * S * SPS, (2 * S + 1) * SPS>(c0, c1, ib, f, jlane, best, bestj);
        n1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq[S], afrag[1][S], S == 0 ? f32x16{0} : n1, 0, 0, 0);
        if constexpr (FOLD) fold_steps<(2 * S + 1) * SPS, (2 * S + 2) * SPS>(c0, c1, ib, f, jlane, best, bestj);
      };
      static_for(kstep, std::make_integer_sequence<int, KSTEPS>{});
      // pin the fold to this stage (its results are otherwise free to sink into a later block)
      if constexpr (FOLD) asm volatile("" : "+v"(best[0]), "+v"(best[1]), "+v"(bestj[0]), "+v"(bestj[1]));
      load_ib(row_c, ib_next);       // norms of the tile just multiplied, for its fold one stage on
    };
    f32x16 xa0, xa1, xb0, xb1;
    f32x4 iba[4], ibb[4];
    auto panel_body = [&](auto buf_c, int p) {
      constexpr int BUF = decltype(buf_c)::value;
      constexpr int R = BUF * kPanel, RN = (BUF ^ 1) * kPanel;
      const int j0 = p * kPanel + jl;
      stage(std::integral_constant<int, R + 32>{}, std::true_type{}, xb0, xb1, xa0, xa1, iba, ibb, j0);
      stage(std::integral_constant<int, R + 64>{}, std::true_type{}, xa0, xa1, xb0, xb1, ibb, iba, j0 + 32);
      stage(std::integral_constant<int, R + 96>{}, std::true_type{}, xb0, xb1, xa0, xa1, iba, ibb, j0 + 64);
      if (p + 1 < n_panels) {
        store_panel(BUF ^ 1, (p + 1) * kPanel);
        if (p + 2 < n_panels) load_panel((p + 2) * kPanel);
        __syncthreads();
        stage(std::integral_constant<int, RN>{}, std::true_type{}, xa0, xa1, xb0, xb1, ibb, iba, j0 + 96);
      } else {
        FoldRegs f;
        fold_steps<0, kFoldSteps>(xb0, xb1, ibb, f, j0 + 96, best, bestj);
      }
    };
    store_panel(0, 0);
    if (n_panels > 1) load_panel(kPanel);
    __syncthreads();
    stage(std::integral_constant<int, 0>{}, std::false_type{}, xa0, xa1, xb0, xb1, ibb, iba, 0);
    for (int p = 0; p < n_panels; p += 2) {
      panel_body(std::integral_constant<int, 0>{}, p);
      if (p + 1 < n_panels) panel_body(std::integral_constant<int, 1>{}, p + 1);
    }
  } else {
  store_panel(0, p_first * kPanel);
  for (int it_p = 0; it_p < n_panels; ++it_p) {
    int p = p_first + it_p;
    if (p >= n_panels) p -= n_panels;
    int p_next = p + 1;
    if (p_next >= n_panels) p_next = 0;
    const int buf = it_p & 1, pbase = p * kPanel;
    if (it_p + 1 < n_panels) load_panel(p_next * kPanel);
    __syncthreads();
    if (wave_active) {
      const int rows_here = min(kPanel, nB - pbase);
      if (rows_here == kPanel) {
        if (buf == 0) compute_tiles(std::integral_constant<int, 0>{}, std::true_type{}, pbase, kPanel);
        else compute_tiles(std::integral_constant<int, 1>{}, std::true_type{}, pbase, kPanel);
      } else {
        if (buf == 0) compute_tiles(std::integral_constant<int, 0>{}, std::false_type{}, pbase, rows_here);
        else compute_tiles(std::integral_constant<int, 1>{}, std::false_type{}, pbase, rows_here);
      }
    }
    if (it_p + 1 < n_panels) store_panel(buf ^ 1, p_next * kPanel);
  }
  }

  // ---- merge the two lane halves of every A row and write ------------------------------------
  if (wave_active) {
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      const float ob = __shfl_xor(best[rt], 32);
      const int oj = __shfl_xor(bestj[rt], 32);
      float b = best[rt];
      int j = bestj[rt];
      if (ob > b || (ob == b && oj < j)) { b = ob; j = oj; }
      const int a = a0 + wave * kRowsPerWave + rt * 32 + col;
      if (half == 0 && a < nA) {
        dst_local[out_base + a] = j;
        score[out_base + a] = b * my_inva[rt];
      }
    }
  }
}

// ---- whole chunks of 64, 128 or 256 tokens (the sizes of the paper's chunk ablation, Sec. 6.4) ----
// A workgroup of match_bf16_kernel owns one chunk; at these sizes it would stage a 128-row panel
// and keep four waves around a block of 32 to 128 rows.  Here a workgroup takes 512 consecutive
// tokens of a sequence, that is 8, 4 or 2 whole chunks: their 256 A rows go through LDS into the
// waves' operand registers, their 256 B rows are normed and parked in LDS in one go, and every
// 32-row tile of A rows is multiplied with the B tiles of its own chunk only (1, 2 or 4 of them).
// Same operand order, same norms and the same fold as match_bf16_kernel: same bits.
constexpr int kSmallTokens = 512;

template <int D>
__global__ __launch_bounds__(kThreads, 2) void match_small_bf16_kernel(
    const __bf16* __restrict__ K, TensorView kv, int seq, int chunk, int n_full, int blocks_per_seq, int total_work,
    int per_xcd, int32_t* __restrict__ dst_local, float* __restrict__ score) {
  constexpr int OCT = D / 8, ROWB = D * 2, KEYSHIFT = (ROWB == 256) ? 0 : 1, KSTEPS = D / 16;
  constexpr int ROWS = kSmallTokens / 2;           // A rows = B rows of a full block
  constexpr int ROWS_PER_PASS = kThreads / OCT, PIECES = ROWS / ROWS_PER_PASS;
  static_assert(ROWS_PER_PASS % (OCT << KEYSHIFT) == 0, "swizzle period");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* rows_lds = smem;                                 // ROWS rows: first the A rows, then the B rows
  float* invb = reinterpret_cast<float*>(smem + ROWS * ROWB);     // 1/|k_j| of the B rows

  const int w = xcd_remap(blockIdx.x, per_xcd);
  if (w >= total_work) return;
  const int sb = w % blocks_per_seq, bh = w / blocks_per_seq;
  const int t0 = sb * kSmallTokens;
  const int nrows = min(kSmallTokens, n_full * chunk - t0) >> 1;  // whole chunks only: a multiple of chunk / 2 >= 32
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int piece = tid % OCT, r0 = tid / OCT;
  const __bf16* Kblk = K + kv.seq_base(bh) + (int64_t)t0 * kv.stride_s + piece * 8;
  auto swz = [](int row, int pc) -> int { return row * ROWB + (((pc ^ (row >> KEYSHIFT)) & (OCT - 1)) << 4); };
  const int lds_piece0 = swz(r0, piece);

  // all loads of the block before the first use; rows past the block's end re-read its last row and are zeroed
  Piece xa[PIECES], xb[PIECES];
#pragma unroll
  for (int it = 0; it < PIECES; ++it) {
    const int r = min(r0 + it * ROWS_PER_PASS, nrows - 1);
    xa[it].u = *reinterpret_cast<const uint4*>(Kblk + (int64_t)(2 * r) * kv.stride_s);
  }
#pragma unroll
  for (int it = 0; it < PIECES; ++it) {
    const int r = min(r0 + it * ROWS_PER_PASS, nrows - 1);
    xb[it].u = *reinterpret_cast<const uint4*>(Kblk + (int64_t)(2 * r + 1) * kv.stride_s);
  }
#pragma unroll
  for (int it = 0; it < PIECES; ++it) {
    if (r0 + it * ROWS_PER_PASS >= nrows) xa[it].u = make_uint4(0, 0, 0, 0);
    *reinterpret_cast<uint4*>(rows_lds + lds_piece0 + it * ROWS_PER_PASS * ROWB) = xa[it].u;
  }
  __syncthreads();
  bf16x8 afrag[2][KSTEPS];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    const int row = wave * kRowsPerWave + rt * 32 + col;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) afrag[rt][s] = *reinterpret_cast<const bf16x8*>(rows_lds + swz(row, 2 * s + half));
  }
  const float my_inva[2] = {inv_norm_of_operand_row<KSTEPS>(afrag[0]), inv_norm_of_operand_row<KSTEPS>(afrag[1])};
  __syncthreads();
#pragma unroll
  for (int it = 0; it < PIECES; ++it) {
    if (r0 + it * ROWS_PER_PASS >= nrows) xb[it].u = make_uint4(0, 0, 0, 0);
    const float ss = row_sum<OCT>(sumsq8(xb[it]));
    *reinterpret_cast<uint4*>(rows_lds + lds_piece0 + it * ROWS_PER_PASS * ROWB) = xb[it].u;
    if (piece == 0) invb[r0 + it * ROWS_PER_PASS] = inv_norm(ss);
  }
  __syncthreads();

  int boff[KSTEPS];
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) boff[s] = swz(col, 2 * s + half);
  const int tiles_per_chunk = chunk >> 6;          // B tiles (= A tiles) of a chunk: 1, 2 or 4
  const int n_src = n_sources(seq, chunk);
  const int64_t out_base = (int64_t)bh * n_src + (t0 >> 1);   // whole chunks before this block: source index = token / 2
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    const int tile = 2 * wave + rt;                // this wave's A tile within the block
    if (tile * 32 >= nrows) break;                 // (uniform over the wave)
    const int first = (tile / tiles_per_chunk) * tiles_per_chunk;   // first B tile of the A tile's chunk
    float best = -INFINITY;
    int bestj = 0;
    for (int tt = 0; tt < tiles_per_chunk; ++tt) {
      const unsigned char* pb = rows_lds + (first + tt) * 32 * ROWB;
      f32x16 acc = {0};
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(pb + boff[s]), afrag[rt][s], acc, 0, 0, 0);
      f32x4 ib[4];
#pragma unroll
      for (int qd = 0; qd < 4; ++qd)
        ib[qd] = *reinterpret_cast<const f32x4*>(invb + (first + tt) * 32 + 4 * half + 8 * qd);
      tile_argmax<false>(acc, ib, tt * 32, half, 32, best, bestj);
    }
    const float ob = __shfl_xor(best, 32);
    const int oj = __shfl_xor(bestj, 32);
    if (ob > best || (ob == best && oj < bestj)) { best = ob; bestj = oj; }
    if (half == 0) {
      const int a = tile * 32 + col;
      dst_local[out_base + a] = bestj;
      score[out_base + a] = best * my_inva[rt];
    }
  }
}

// ---- persistent streaming kernel: bf16, dim 128, whole chunks of 1024 or 2048 tokens -----------
// One workgroup per CU walks a contiguous range of items: (sequence, chunk, block of 512 A rows),
// one block per 1024-token chunk, two per 2048-token chunk (each against all of the chunk's B
// rows: TILES = 16 or 32 B tiles per item).  While an item is
// matched, the NEXT item's A rows arrive in a 128 KiB LDS area (one 32-row pass per stage) and the
// B rows stream through a ring of three 32-row tiles (one tile per stage, loaded four stages
// ahead into registers, normed on the way into LDS); at 1024 tokens the two row streams are just
// the even and odd tokens of one contiguous walk through memory.  At an item boundary the A
// operands are re-read from LDS, so no global-memory latency is exposed between items.  Every stage folds
// tile q while the MFMAs of tile q+1 run (see the pipelined loop of match_bf16_kernel).
constexpr int kStreamBlock = 512;       // A rows per item
constexpr int kStreamThreads = 512;
constexpr int kStreamTile = 32;
constexpr int kStreamSlots = 3;
constexpr size_t kStreamLds = (size_t)kStreamBlock * 256 + kStreamSlots * kStreamTile * 256 +
                              kStreamSlots * kStreamTile * sizeof(float);

template <int TILES>
__global__ __launch_bounds__(kStreamThreads, 1) void match_stream_bf16_kernel(
    const __bf16* __restrict__ K, TensorView kv, int seq, int n_chunks, int total_items,
    int32_t* __restrict__ dst_local, float* __restrict__ score) {
  constexpr int ROWB = 256, KSTEPS = 8, HALF = kStreamBlock, APASSES = HALF / kStreamTile;
  constexpr int CHUNK = 2 * TILES * kStreamTile;   // tokens per chunk
  constexpr int AB = TILES / APASSES;              // A blocks (items) per chunk
  constexpr int NA = 4 / AB;                       // A passes in flight (one is handed over every AB stages)
  constexpr int TILEB = kStreamTile * ROWB;
  static_assert(TILES == 16 || TILES == 32, "chunks of 1024 or 2048 tokens");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* abuf = smem;                                    // A rows of the next item
  unsigned char* ring = smem + HALF * ROWB;                      // kStreamSlots B tiles
  float* invb = reinterpret_cast<float*>(ring + kStreamSlots * TILEB);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int piece = tid & 15, r0 = tid >> 4;                     // this thread's 16 bytes of a 32-row pass
  const int lds_piece0 = r0 * ROWB + ((piece ^ (r0 & 15)) << 4);
  const int first = (int)((int64_t)blockIdx.x * total_items / gridDim.x);
  const int last = (int)((int64_t)(blockIdx.x + 1) * total_items / gridDim.x);
  if (first >= last) return;
  const int n_src = n_sources(seq, CHUNK);
  const int64_t pass_pitch = 2 * kStreamTile * kv.stride_s;      // 32 A rows (or B rows) further on

  // Addresses = a workgroup-uniform pass pointer + this thread's fixed offset inside a pass (row
  // r0, its 16-byte piece), so the walks below cost scalar instructions only.  a_ptr / b_ptr: A row
  // 0 of an item's block / B row 0 of its chunk (item clamped to the range).
  const uint32_t toff = (uint32_t)(2 * r0 * kv.stride_s + piece * 8) * 2u;   // bytes
  auto chunk_ptr = [&](int item, int& ab) -> const __bf16* {
    item = min(item, last - 1);
    const int cg = item / AB;
    ab = item - cg * AB;
    const int bh = cg / n_chunks, g = cg - bh * n_chunks;
    return K + kv.seq_base(bh) + (int64_t)g * CHUNK * kv.stride_s;
  };
  auto a_ptr = [&](int item) -> const __bf16* {
    int ab;
    const __bf16* c = chunk_ptr(item, ab);
    return c + (int64_t)ab * 2 * HALF * kv.stride_s;
  };
  auto b_ptr = [&](int item) -> const __bf16* {
    int ab;
    return chunk_ptr(item, ab) + kv.stride_s;
  };
  auto ld = [&](const __bf16* pass) {
    Piece x;
    x.u = *reinterpret_cast<const uint4*>(reinterpret_cast<const unsigned char*>(pass) + toff);
    return x;
  };
  auto put_b = [&](int slot, const Piece& x) {                   // B piece + its row's norm (all 16
    const float ss = row_sum<16>(sumsq8(x));                     // lanes of a row store the same value)
    *reinterpret_cast<uint4*>(ring + slot * TILEB + lds_piece0) = x.u;
    invb[slot * kStreamTile + r0] = inv_norm(ss);
  };

  // ---- prologue: A rows of the first item, B tiles 0 and 1, four stages of each stream in flight
  Piece sb[4], sa[NA];
  const __bf16 *pB, *pA;                 // next pass each stream loads: B six tiles, A four stages ahead
  {
    const __bf16* a0 = a_ptr(first);
    const __bf16* b0p = b_ptr(first);
    const __bf16* a1 = a_ptr(first + 1);
    Piece xa[APASSES];
#pragma unroll
    for (int t = 0; t < APASSES; ++t) xa[t] = ld(a0 + t * pass_pitch);
    const Piece b0 = ld(b0p);
    const Piece b1 = ld(b0p + pass_pitch);
#pragma unroll
    for (int u = 0; u < 4; ++u) sb[u] = ld(b0p + (u + 2) * pass_pitch);
#pragma unroll
    for (int u = 0; u < NA; ++u) sa[u] = ld(a1 + u * pass_pitch);
    pB = b0p + 6 * pass_pitch;
    pA = a1 + NA * pass_pitch;
#pragma unroll
    for (int t = 0; t < APASSES; ++t) *reinterpret_cast<uint4*>(abuf + t * TILEB + lds_piece0) = xa[t].u;
    put_b(0, b0);
    put_b(1, b1);
  }
  __syncthreads();
  bf16x8 afrag[2][KSTEPS];
  float my_inva[2];
  auto load_afrag = [&](float (&inva)[2]) {
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      const int row = wave * kRowsPerWave + rt * 32 + col;
#pragma unroll
      for (int s = 0; s < KSTEPS; ++s)
        afrag[rt][s] = *reinterpret_cast<const bf16x8*>(abuf + row * ROWB + ((((2 * s + half) ^ row) & 15) << 4));
    }
    inva[0] = inv_norm_of_operand_row<KSTEPS>(afrag[0]);
    inva[1] = inv_norm_of_operand_row<KSTEPS>(afrag[1]);
  };
  load_afrag(my_inva);
  __syncthreads();

  int boff[KSTEPS];
#pragma unroll
  for (int s = 0; s < KSTEPS; ++s) boff[s] = col * ROWB + ((((2 * s + half) ^ col) & 15) << 4);
  const int jl = 4 * half;
  const float* ib_lane = invb + jl;
  float best[2] = {-INFINITY, -INFINITY};
  int bestj[2] = {0, 0};

  // MFMAs of the tile in `slot` into (n0, n1); with FOLD, the tile held in (c0, c1) is folded behind
  // them.  The first two B fragments were read at the end of the stage before (the tile is complete
  // in LDS by then), the next tile's are read here, so no LDS latency follows the barrier.
  bf16x8 pre[2];
  auto prefetch = [&](int slot) {
    pre[0] = *reinterpret_cast<const bf16x8*>(ring + slot * TILEB + boff[0]);
    pre[1] = *reinterpret_cast<const bf16x8*>(ring + slot * TILEB + boff[1]);
  };
  auto stage = [&](int slot, int slot_next, auto fold_c, f32x16& n0, f32x16& n1, f32x16& c0, f32x16& c1,
                   const f32x4 (&ib)[4], f32x4 (&ib_next)[4], int jlane) {
    constexpr bool FOLD = decltype(fold_c)::value;
    constexpr int SPS = (kFoldSteps + 2 * KSTEPS - 1) / (2 * KSTEPS);
    const unsigned char* pb = ring + slot * TILEB;
    bf16x8 bq[KSTEPS];
    bq[0] = pre[0];
    bq[1] = pre[1];
    FoldRegs f;
    auto kstep = [&](auto s_c) {
      constexpr int S = decltype(s_c)::value;
      if constexpr (S + 2 < KSTEPS) bq[S + 2] = *reinterpret_cast<const bf16x8*>(pb + boff[S + 2]);
      n0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq[S], afrag[0][S], S == 0 ? f32x16{0} : n0, 0, 0, 0);
      if constexpr (FOLD) fold_steps<2 * S * SPS, (2 * S + 1) * SPS>(c0, c1, ib, f, jlane, best, bestj);
      n1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq[S], afrag[1][S], S == 0 ? f32x16{0} : n1, 0, 0, 0);
      if constexpr (FOLD) fold_steps<(2 * S + 1) * SPS, (2 * S + 2) * SPS>(c0, c1, ib, f, jlane, best, bestj);
    };
    static_for(kstep, std::make_integer_sequence<int, KSTEPS>{});
    // pin the fold to this stage (its results are otherwise free to sink into a later block)
    if constexpr (FOLD) asm volatile("" : "+v"(best[0]), "+v"(best[1]), "+v"(bestj[0]), "+v"(bestj[1]));
#pragma unroll
    for (int qd = 0; qd < 4; ++qd)      // norms of the tile just multiplied, for its fold one stage on
      ib_next[qd] = *reinterpret_cast<const f32x4*>(ib_lane + slot * kStreamTile + 8 * qd);
    prefetch(slot_next);
  };

  f32x16 xa0, xa1, xb0, xb1;
  f32x4 iba[4], ibb[4];
  prefetch(0);
  stage(0, 1, std::false_type{}, xa0, xa1, xb0, xb1, ibb, iba, 0);
  int rs = 1, ws = 2;                    // ring slots: tile q+1 is read, tile q+2 written, in stage q
  for (int item = first; item < last; ++item) {
    // where the two streams continue once they run off their current item: B after the item's last
    // tile (loaded six stages ahead), A after the next item's last pass (loaded four stages ahead)
    const __bf16* wrapB = b_ptr(item + 1);
    const __bf16* wrapA = a_ptr(item + 2);
    float next_inva[2] = {my_inva[0], my_inva[1]};
    for (int t0 = 0; t0 < TILES; t0 += 4) {
      // stage t: hand over the passes loaded four stages ago, refill their registers (no branch:
      // the four stages of this body stay one straight-line block), then compute
      auto feed = [&](auto u_c) {
        constexpr int U = decltype(u_c)::value;
        const int t = t0 + U;
        put_b(ws, sb[U]);
        sb[U] = ld(pB);
        pB = (t == TILES - 7) ? wrapB : pB + pass_pitch;
        if constexpr (U % AB == 0) {     // an A pass of the next item every AB stages
          *reinterpret_cast<uint4*>(abuf + (t / AB) * TILEB + lds_piece0) = sa[U / AB].u;
          sa[U / AB] = ld(pA);
          pA = (t == (APASSES - 1 - NA) * AB) ? wrapA : pA + pass_pitch;
        }
        __syncthreads();
      };
      auto turn = [&] {
        rs = (rs == kStreamSlots - 1) ? 0 : rs + 1;
        ws = (ws == kStreamSlots - 1) ? 0 : ws + 1;
      };
      const int j0 = t0 * kStreamTile + jl;
      feed(std::integral_constant<int, 0>{});
      stage(rs, ws, std::true_type{}, xb0, xb1, xa0, xa1, iba, ibb, j0);
      turn();
      feed(std::integral_constant<int, 1>{});
      stage(rs, ws, std::true_type{}, xa0, xa1, xb0, xb1, ibb, iba, j0 + 32);
      turn();
      feed(std::integral_constant<int, 2>{});
      stage(rs, ws, std::true_type{}, xb0, xb1, xa0, xa1, iba, ibb, j0 + 64);
      turn();
      feed(std::integral_constant<int, 3>{});
      if (t0 + 4 == TILES && item + 1 < last) {   // the next tile belongs to the next item: its A
        load_afrag(next_inva);                    // operands (this item's 1/|k_i| is still needed)
        __syncthreads();                          // abuf may now take the rows of the item after that
      }
      stage(rs, ws, std::true_type{}, xa0, xa1, xb0, xb1, ibb, iba, j0 + 96);
      turn();
    }
    // the item's last tile is folded: write its matches
    const int cg = item / AB, ab = item - cg * AB;
    const int bh = cg / n_chunks, g = cg - bh * n_chunks;
    const int64_t out_base = (int64_t)bh * n_src + (int64_t)g * (CHUNK / 2) + ab * HALF;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      const float ob = __shfl_xor(best[rt], 32);
      const int oj = __shfl_xor(bestj[rt], 32);
      float b = best[rt];
      int j = bestj[rt];
      if (ob > b || (ob == b && oj < j)) { b = ob; j = oj; }
      const int a = wave * kRowsPerWave + rt * 32 + col;
      if (half == 0) {
        dst_local[out_base + a] = j;
        score[out_base + a] = b * my_inva[rt];
      }
      best[rt] = -INFINITY;
      bestj[rt] = 0;
      my_inva[rt] = next_inva[rt];
    }
  }
}

// ---- fp32 keys: plain FMA, LDS tiles; a correctness path, not a roofline one -------------------
constexpr int kF32ARows = 64, kF32BRows = 32, kF32MaxD = 128;

constexpr int kF32MaxBlocks = 2048 / 8 + 2;   // block-table entries of a chunk (paged input: blocks of 8 tokens or more)
template <bool PAGED>
__global__ __launch_bounds__(kThreads) void match_f32_kernel(
    const float* __restrict__ K, TensorView kv, int dim, int seq, int chunk, int n_chunks,
    int a_blocks, int32_t* __restrict__ dst_local, float* __restrict__ score, PagedSide paged) {
  __shared__ float As[kF32ARows][kF32MaxD + 1];
  __shared__ float Bs[kF32BRows][kF32MaxD + 1];
  __shared__ float inva[kF32ARows], invb[kF32BRows];
  __shared__ int32_t s_rb[PAGED ? kF32MaxBlocks : 1];
  const int w = blockIdx.x;
  const int ab = w % a_blocks, g = (w / a_blocks) % n_chunks, bh = w / (a_blocks * n_chunks);
  const int g0 = g * chunk, L = min(chunk, seq - g0);
  const int nA = (L + 1) >> 1, nB = L >> 1, a0 = ab * kF32ARows;
  if (a0 >= nA) return;
  const int tid = threadIdx.x;
  const int n_src = n_sources(seq, chunk);
  const int64_t out_base = (int64_t)bh * n_src + (int64_t)g * (chunk >> 1);
  if (nB == 0) {
    if (tid == 0) { dst_local[out_base] = -1; score[out_base] = 0.f; }
    return;
  }
  const float* Kseq = PAGED ? K : K + kv.seq_base(bh) + (int64_t)g0 * kv.stride_s;
  RowBases rows{};
  const int u0 = paged.tok0 + g0;
  if (PAGED) {
    rows = stage_row_bases(s_rb, paged, bh / kv.heads, bh % kv.heads, kv.heads, u0, u0 + L - 1, tid, kThreads);
    __syncthreads();
  }
  auto tok_ptr = [&](int u) -> const float* {
    if (PAGED) return K + (int64_t)rows.row(u0 + u) * dim;
    return Kseq + (int64_t)u * kv.stride_s;
  };
  for (int e = tid; e < kF32ARows * dim; e += kThreads) {
    const int row = e / dim, k = e % dim, a = a0 + row;
    As[row][k] = (a < nA) ? tok_ptr(2 * a)[k] : 0.f;
  }
  __syncthreads();
  if (tid < kF32ARows) {
    float ss = 0.f;
    for (int k = 0; k < dim; ++k) ss = fmaf(As[tid][k], As[tid][k], ss);
    inva[tid] = inv_norm(ss);
  }
  const int r = tid >> 2, q = tid & 3;
  float best = -INFINITY;
  int bestj = 0;
  for (int pbase = 0; pbase < nB; pbase += kF32BRows) {
    __syncthreads();
    for (int e = tid; e < kF32BRows * dim; e += kThreads) {
      const int row = e / dim, k = e % dim, j = pbase + row;
      Bs[row][k] = (j < nB) ? tok_ptr(2 * j + 1)[k] : 0.f;
    }
    __syncthreads();
    if (tid < kF32BRows) {
      float ss = 0.f;
      for (int k = 0; k < dim; ++k) ss = fmaf(Bs[tid][k], Bs[tid][k], ss);
      invb[tid] = inv_norm(ss);
    }
    __syncthreads();
    float acc[kF32BRows / 4];
#pragma unroll
    for (int m = 0; m < kF32BRows / 4; ++m) acc[m] = 0.f;
    for (int k = 0; k < dim; ++k) {
      const float a = As[r][k];
#pragma unroll
      for (int m = 0; m < kF32BRows / 4; ++m) acc[m] = fmaf(a, Bs[q + 4 * m][k], acc[m]);
    }
#pragma unroll
    for (int m = 0; m < kF32BRows / 4; ++m) {
      const int jl = q + 4 * m, j = pbase + jl;
      const float s = acc[m] * invb[jl];
      if (j < nB && s > best) { best = s; bestj = j; }
    }
  }
#pragma unroll
  for (int m = 1; m < 4; m <<= 1) {
    const float ob = __shfl_xor(best, m);
    const int oj = __shfl_xor(bestj, m);
    if (ob > best || (ob == best && oj < bestj)) { best = ob; bestj = oj; }
  }
  const int a = a0 + r;
  if (q == 0 && a < nA) {
    dst_local[out_base + a] = bestj;
    score[out_base + a] = best * inva[r];
  }
}

__global__ void dst_positions_kernel(const int32_t* __restrict__ dst_local, int32_t* __restrict__ dst_pos,
                                     int n_src, int chunk, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  const int i = (int)(e % n_src);
  const int g = i / (chunk >> 1);
  const int j = dst_local[e];
  dst_pos[e] = (j < 0) ? -1 : g * chunk + 2 * j + 1;
}

template <int D, int NW, bool PAGED>
hipError_t launch_match_bf16_nw(const void* K, TensorView kv, int n_bh, int seq, int chunk,
                                int32_t* dst_local, float* score, hipStream_t st, PagedSide paged, int g_first = 0) {
  constexpr int ABLOCK = NW * kRowsPerWave;
  // staging area + inverse norms of two panels (+ PAGED: the pool rows of a chunk's blocks, 8 tokens or more each)
  constexpr size_t lds = (size_t)(ABLOCK > 2 * kPanel ? ABLOCK : 2 * kPanel) * D * 2 + 2 * kPanel * sizeof(float) +
                         (PAGED ? (2048 / 8 + 2) * sizeof(int32_t) : 0);
  static KernelSetup setup;
  if (hipError_t e = kernel_setup(reinterpret_cast<const void*>(&match_bf16_kernel<D, NW, PAGED>), lds, setup); e != hipSuccess)
    return e;
  const int n_chunks = div_up(seq, chunk) - g_first;     // chunks g_first .. last
  const int a_blocks = div_up(chunk / 2, ABLOCK);
  const int64_t total = (int64_t)n_bh * n_chunks * a_blocks;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  const int per_xcd = div_up((int)total, 8);
  ScopedTimer t("match_bf16", st);
  hipLaunchKernelGGL((match_bf16_kernel<D, NW, PAGED>), dim3(per_xcd * 8), dim3(NW * 64), lds, st,
                     static_cast<const __bf16*>(K), kv, seq, chunk, n_chunks, g_first, a_blocks, (int)total,
                     per_xcd, dst_local, score, paged);
  return hipGetLastError();
}

// Chunks of 64, 128 or 256 tokens: the whole chunks of every sequence in blocks of 512 tokens, then the
// ragged tail chunk (if any) with the one-chunk-per-workgroup kernel.
template <int D>
hipError_t launch_match_small(const void* K, TensorView kv, int n_bh, int seq, int chunk, int32_t* dst_local,
                              float* score, hipStream_t st) {
  constexpr size_t lds = (size_t)(kSmallTokens / 2) * D * 2 + (kSmallTokens / 2) * sizeof(float);
  static KernelSetup setup;
  if (hipError_t e = kernel_setup(reinterpret_cast<const void*>(&match_small_bf16_kernel<D>), lds, setup); e != hipSuccess)
    return e;
  const int n_full = seq / chunk;
  const int blocks_per_seq = div_up(n_full * chunk, kSmallTokens);
  const int64_t total = (int64_t)n_bh * blocks_per_seq;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  const int per_xcd = div_up((int)total, 8);
  {
    ScopedTimer t("match_bf16", st);
    hipLaunchKernelGGL((match_small_bf16_kernel<D>), dim3(per_xcd * 8), dim3(kThreads), lds, st,
                       static_cast<const __bf16*>(K), kv, seq, chunk, n_full, blocks_per_seq, (int)total, per_xcd,
                       dst_local, score);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  }
  if (seq % chunk == 0) return hipSuccess;
  return launch_match_bf16_nw<D, 4, false>(K, kv, n_bh, seq, chunk, dst_local, score, st, PagedSide{}, n_full);
}

// Whole 1024- or 2048-token chunks of 128-dim keys: the persistent kernel, one workgroup per CU.
template <int TILES>
hipError_t launch_match_stream(const void* K, TensorView kv, int n_bh, int seq, int32_t* dst_local,
                               float* score, hipStream_t st) {
  static KernelSetup setup;
  int n_cu = 0;
  if (hipError_t e = kernel_setup(reinterpret_cast<const void*>(&match_stream_bf16_kernel<TILES>), kStreamLds, setup, &n_cu);
      e != hipSuccess)
    return e;
  constexpr int CHUNK = 2 * TILES * kStreamTile;
  const int n_chunks = seq / CHUNK;
  const int64_t total = (int64_t)n_bh * n_chunks * (TILES / 16);
  if (total > (1 << 30)) return hipErrorInvalidValue;
  const int grid = (int)(total < n_cu ? total : n_cu);
  ScopedTimer t("match_bf16", st);
  hipLaunchKernelGGL(match_stream_bf16_kernel<TILES>, dim3(grid), dim3(kStreamThreads), kStreamLds, st,
                     static_cast<const __bf16*>(K), kv, seq, n_chunks, (int)total, dst_local, score);
  return hipGetLastError();
}

template <int D>
hipError_t launch_match_bf16(const void* K, TensorView kv, int n_bh, int seq, int chunk,
                             int32_t* dst_local, float* score, hipStream_t st, PagedSide paged) {
  if (paged.table) {
    if (chunk > 512) return launch_match_bf16_nw<D, 8, true>(K, kv, n_bh, seq, chunk, dst_local, score, st, paged);
    return launch_match_bf16_nw<D, 4, true>(K, kv, n_bh, seq, chunk, dst_local, score, st, paged);
  }
  if (chunk > 512) return launch_match_bf16_nw<D, 8, false>(K, kv, n_bh, seq, chunk, dst_local, score, st, paged);
  if ((chunk == 64 || chunk == 128 || chunk == 256) && seq >= chunk)
    return launch_match_small<D>(K, kv, n_bh, seq, chunk, dst_local, score, st);
  return launch_match_bf16_nw<D, 4, false>(K, kv, n_bh, seq, chunk, dst_local, score, st, paged);
}

}  // namespace

hipError_t launch_match(const void* K, int dtype, int dim, TensorView kv, int n_bh, int seq,
                        int chunk, int32_t* dst_local, float* score, hipStream_t st, PagedSide paged) {
  if (paged.table && paged.shift < 3) return hipErrorInvalidValue;   // the kernels' LDS tables hold blocks of 8 tokens or more
  if (dtype == CKV_BF16) {
    // (the persistent streaming kernel walks memory with fixed pitches: strided tensors only)
    if (!paged.table && dim == 128 && (chunk == 1024 || chunk == 2048) && seq % chunk == 0 && seq > 0 && kv.stride_s <= (1 << 22))
      return chunk == 1024 ? launch_match_stream<16>(K, kv, n_bh, seq, dst_local, score, st)
                           : launch_match_stream<32>(K, kv, n_bh, seq, dst_local, score, st);
    if (dim == 128) return launch_match_bf16<128>(K, kv, n_bh, seq, chunk, dst_local, score, st, paged);
    if (dim == 64) return launch_match_bf16<64>(K, kv, n_bh, seq, chunk, dst_local, score, st, paged);
    return hipErrorInvalidValue;
  }
  if (dim > kF32MaxD) return hipErrorInvalidValue;
  const int n_chunks = div_up(seq, chunk);
  const int a_blocks = div_up(chunk / 2, kF32ARows);
  const int64_t total = (int64_t)n_bh * n_chunks * a_blocks;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  ScopedTimer t("match_f32", st);
  if (paged.table)
    hipLaunchKernelGGL(match_f32_kernel<true>, dim3((int)total), dim3(kThreads), 0, st,
                       static_cast<const float*>(K), kv, dim, seq, chunk, n_chunks, a_blocks, dst_local, score, paged);
  else
    hipLaunchKernelGGL(match_f32_kernel<false>, dim3((int)total), dim3(kThreads), 0, st,
                       static_cast<const float*>(K), kv, dim, seq, chunk, n_chunks, a_blocks, dst_local, score, paged);
  return hipGetLastError();
}

hipError_t launch_dst_positions(const int32_t* dst_local, int32_t* dst_pos, int n_bh, int seq,
                                int chunk, hipStream_t st) {
  const int n_src = n_sources(seq, chunk);
  const int64_t total = (int64_t)n_bh * n_src;
  ScopedTimer t("dst_positions", st);
  hipLaunchKernelGGL(dst_positions_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     dst_local, dst_pos, n_src, chunk, total);
  return hipGetLastError();
}

}  // namespace ckv
