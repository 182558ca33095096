// Similarity + matching stage of Chunked Soft Matching (Sec. 5.2, Eq. 2) for gfx950.
//
// Per chunk of L tokens: A = tokens at even offsets (sources), B = odd offsets (destinations).
// For every A token i:  j*(i) = argmax_j  k_i.k_j / (|k_i||k_j|)  (lowest j on ties) and that
// maximum.  The |A| x |B| similarity matrix lives only in MFMA accumulators.
//
// bf16 kernel: one workgroup = (sequence, chunk, block of A rows), 64 A rows per wave; 8 waves
// (512 A rows: a whole 1024-token chunk) for chunks above 512 tokens, 4 waves otherwise.  The
// A rows are staged once through LDS into registers in MFMA operand order; the chunk's B rows
// stream through two LDS panels of 128 rows (global -> registers -> LDS, one barrier per panel).
// Inverse norms come from the same bytes (v_dot2 on the packed pairs): the B rows' while they
// are staged, the A rows' from the operand registers.  The MFMA computes
// S^T (B index on the M side) so that a lane's 16 accumulators of a 32x32 tile all belong to ONE
// A row: the running maximum costs one multiply (by 1/|k_j|) and half a max3 per element, and the
// exact index is only resolved for tiles that raise some lane's maximum.
#include <type_traits>

#include "ckv_internal.h"
#include "ckv_device.h"

namespace ckv {
namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerWave = 64;                 // two 32-row MFMA tiles
constexpr int kPanel = 128;                      // B rows per LDS panel

// NW waves x 64 A rows per workgroup: 4 waves (two workgroups per CU) for chunks of up to 512 tokens,
// 8 waves (one workgroup per CU) for larger chunks, so that the B rows of a 1024-token chunk are
// fetched, normed and written to LDS once instead of once per 256 A rows.
template <int D, int NW>
__global__ __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) void match_bf16_kernel(
    const __bf16* __restrict__ K, TensorView kv, int seq, int chunk, int n_chunks, int a_blocks,
    int total_work, int per_xcd, int32_t* __restrict__ dst_local, float* __restrict__ score) {
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

  const int w = xcd_remap(blockIdx.x, per_xcd);
  if (w >= total_work) return;
  const int ab = w % a_blocks;
  const int g = (w / a_blocks) % n_chunks;
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
  const __bf16* Kseq = K + kv.seq_base(bh) + (int64_t)g0 * kv.stride_s;

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
        stage[it].u = *reinterpret_cast<const uint4*>(Bcol + j * row_pitch);
      }
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
  const int p_first = min(a0 / kPanel, n_panels - 1);
  {
    constexpr int APIECES = ABLOCK * OCT / THREADS;
    Piece xa[APIECES];
#pragma unroll
    for (int it = 0; it < APIECES; ++it) {
      const int a = min(a0 + r0 + it * ROWS_PER_PASS, nA - 1);
      xa[it].u = *reinterpret_cast<const uint4*>(Kseq + (int64_t)(2 * a) * kv.stride_s + piece * 8);
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

// ---- fp32 keys: plain FMA, LDS tiles; a correctness path, not a roofline one -------------------
constexpr int kF32ARows = 64, kF32BRows = 32, kF32MaxD = 128;

__global__ __launch_bounds__(kThreads) void match_f32_kernel(
    const float* __restrict__ K, TensorView kv, int dim, int seq, int chunk, int n_chunks,
    int a_blocks, int32_t* __restrict__ dst_local, float* __restrict__ score) {
  __shared__ float As[kF32ARows][kF32MaxD + 1];
  __shared__ float Bs[kF32BRows][kF32MaxD + 1];
  __shared__ float inva[kF32ARows], invb[kF32BRows];
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
  const float* Kseq = K + kv.seq_base(bh) + (int64_t)g0 * kv.stride_s;
  for (int e = tid; e < kF32ARows * dim; e += kThreads) {
    const int row = e / dim, k = e % dim, a = a0 + row;
    As[row][k] = (a < nA) ? Kseq[(int64_t)(2 * a) * kv.stride_s + k] : 0.f;
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
      Bs[row][k] = (j < nB) ? Kseq[(int64_t)(2 * j + 1) * kv.stride_s + k] : 0.f;
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

template <int D, int NW>
hipError_t launch_match_bf16_nw(const void* K, TensorView kv, int n_bh, int seq, int chunk,
                                int32_t* dst_local, float* score, hipStream_t st) {
  constexpr int ABLOCK = NW * kRowsPerWave;
  constexpr size_t lds = (size_t)(ABLOCK > 2 * kPanel ? ABLOCK : 2 * kPanel) * D * 2 + 2 * kPanel * sizeof(float);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&match_bf16_kernel<D, NW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int n_chunks = div_up(seq, chunk);
  const int a_blocks = div_up(chunk / 2, ABLOCK);
  const int64_t total = (int64_t)n_bh * n_chunks * a_blocks;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  const int per_xcd = div_up((int)total, 8);
  ScopedTimer t("match_bf16", st);
  hipLaunchKernelGGL((match_bf16_kernel<D, NW>), dim3(per_xcd * 8), dim3(NW * 64), lds, st,
                     static_cast<const __bf16*>(K), kv, seq, chunk, n_chunks, a_blocks, (int)total,
                     per_xcd, dst_local, score);
  return hipGetLastError();
}

template <int D>
hipError_t launch_match_bf16(const void* K, TensorView kv, int n_bh, int seq, int chunk,
                             int32_t* dst_local, float* score, hipStream_t st) {
  if (chunk > 512) return launch_match_bf16_nw<D, 8>(K, kv, n_bh, seq, chunk, dst_local, score, st);
  return launch_match_bf16_nw<D, 4>(K, kv, n_bh, seq, chunk, dst_local, score, st);
}

}  // namespace

hipError_t launch_match(const void* K, int dtype, int dim, TensorView kv, int n_bh, int seq,
                        int chunk, int32_t* dst_local, float* score, hipStream_t st) {
  if (dtype == CKV_BF16) {
    if (dim == 128) return launch_match_bf16<128>(K, kv, n_bh, seq, chunk, dst_local, score, st);
    if (dim == 64) return launch_match_bf16<64>(K, kv, n_bh, seq, chunk, dst_local, score, st);
    return hipErrorInvalidValue;
  }
  if (dim > kF32MaxD) return hipErrorInvalidValue;
  const int n_chunks = div_up(seq, chunk);
  const int a_blocks = div_up(chunk / 2, kF32ARows);
  const int64_t total = (int64_t)n_bh * n_chunks * a_blocks;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  ScopedTimer t("match_f32", st);
  hipLaunchKernelGGL(match_f32_kernel, dim3((int)total), dim3(kThreads), 0, st,
                     static_cast<const float*>(K), kv, dim, seq, chunk, n_chunks, a_blocks, dst_local,
                     score);
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
