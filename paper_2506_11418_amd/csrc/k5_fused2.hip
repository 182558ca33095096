// Two clustering rounds in one pass over HBM (Algorithm 1's loop after prefill, for the common
// schedule whose first round merges every edge, r = 1).
//
// With r = 1 a round-0 chunk of c tokens always keeps exactly its c/2 B tokens, so the next
// round's chunk of c tokens is the output of two adjacent round-0 chunks: a "super-chunk" of 2c
// input tokens is a closed unit for both rounds.  One workgroup (8 waves) takes a super-chunk:
//   M0  similarity + argmax of both round-0 chunks (MFMA, as the stand-alone matching kernel);
//   B0  member lists of the round-0 clusters (LDS);
//   G0  the round-0 centroid KEYS are produced on chip: the next round's B rows go to LDS, its A
//       rows straight into MFMA operand registers; values are not touched;
//   M1  similarity + argmax of the round-1 chunk from those registers and LDS;
//   B1  top-r selection, member lists and compaction of round 1 (LDS);
//   E   every output row is gathered from the ORIGINAL keys and values: a round-0 centroid is
//       rebuilt (same fp32 order, same single rounding to bf16 as a stand-alone round) and folded
//       into its round-1 cluster.  Each input row is read once here; nothing intermediate is
//       written to memory.
// Results are bit-identical to running the two rounds one after the other.
#include <type_traits>

#include "ckv_internal.h"
#include "ckv_device.h"

namespace ckv {
namespace {

constexpr int kC = 1024;            // chunk size this kernel is built for
constexpr int kH = kC / 2;          // A (= B) tokens per chunk; also A' (= B') rows of round 1
constexpr int kD = 128;
constexpr int kOct = kD / 8;        // 16-byte pieces per row
constexpr int kRowB = kD * 2;       // bytes per row
constexpr int kKSteps = kD / 16;
constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kSortMax = 8;

// LDS map (bytes)
constexpr int kOffR = 0;                         // 128 KiB: staged rows (swizzled), later round-1 tables
constexpr int kOffInvB = kOffR + kH * kRowB;     // float[512]
constexpr int kOffDst0 = kOffInvB + kH * 4;      // int16[1024]: partner (B index in its chunk) of source s
constexpr int kOffCnt0 = kOffDst0 + 2 * kH * 2;  // int32[1024]: merged sources per round-0 centroid
constexpr int kOffStart0 = kOffCnt0 + 2 * kH * 4;  // int16[1024]
constexpr int kOffMem0 = kOffStart0 + 2 * kH * 2;  // int16[1024]: A index (in its chunk) of members
constexpr int kOffInvA = kOffMem0 + 2 * kH * 2;    // float[512]: 1/|k| of the round-1 A rows
constexpr int kOffDst1 = kOffInvA + kH * 4;    // int16[512]: kept partner of round-1 source or -1
constexpr int kOffScore1 = kOffDst1 + kH * 2;      // float[512]
constexpr int kOffWave = kOffScore1 + kH * 4;      // int[16]
constexpr int kLdsBytes = kOffWave + 64;
// tables that live in R once it is free
constexpr int kOffFill0 = kOffR;                   // int32[1024] (B0 only)
constexpr int kOffCnt1 = kOffR;                    // int32[512]
constexpr int kOffFill1 = kOffCnt1 + kH * 4;       // int32[512]
constexpr int kOffStart1 = kOffFill1 + kH * 4;     // int16[512]
constexpr int kOffMem1 = kOffStart1 + kH * 2;      // int16[512]
constexpr int kOffLout1 = kOffMem1 + kH * 2;       // int16[1024]
constexpr int kOffSrco1 = kOffLout1 + 2 * kH * 2;  // int16[1024]

__device__ __forceinline__ int swz(int row, int piece) { return row * kRowB + (((piece ^ row) & (kOct - 1)) << 4); }

__device__ inline int block_exclusive_scan8(int v, int* s_wave_tot) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(inc, d);
    if (lane >= d) inc += o;
  }
  if (lane == 63) s_wave_tot[wave] = inc;
  __syncthreads();
  int base = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w)
    if (w < wave) base += s_wave_tot[w];
  __syncthreads();
  return base + inc - v;
}

struct Ctx {
  const __bf16* Ksc;       // first key / value row of the super-chunk (workgroup-uniform)
  const __bf16* Vsc;
  const int32_t* dseq;     // degrees of the super-chunk's tokens or nullptr
  uint32_t row_bytes;      // bytes between consecutive tokens
  uint32_t lane_off;       // byte offset of this lane's 16-byte piece inside a row
  const int32_t* cnt0;
  const int16_t* start0;
  const int16_t* mem0;
};

// token (within the super-chunk) of round-0 centroid ip and of its q-th merged source
__device__ __forceinline__ int base_token(int ip) { return ((ip >> 9) << 10) + 2 * (ip & (kH - 1)) + 1; }
__device__ __forceinline__ int member_token(int ip, int a) { return ((ip >> 9) << 10) + 2 * a; }

// One 16-byte piece of the round-0 centroid ip, rounded to bf16 exactly as a stand-alone round
// would store it.  Split in two steps so that a caller can put the loads of several centroids in
// flight before consuming any: issue starts the loads of the centroid's own row and of its first
// merged source (keys, and values when WITH_V), finish does the arithmetic (further sources,
// rare, are loaded there).
template <bool WITH_V>
struct CentroidLoad {
  uint4 kb, k0, vb, v0;
  int db, d0, nm, st, ip;
};

template <bool WITH_V>
__device__ __forceinline__ CentroidLoad<WITH_V> centroid_issue(const Ctx& c, int ip) {
  CentroidLoad<WITH_V> L;
  L.ip = ip;
  L.nm = c.cnt0[ip];
  L.st = c.start0[ip];
  const int tb = base_token(ip);
  const int t0 = L.nm > 0 ? member_token(ip, c.mem0[L.st]) : tb;   // no source: same row again (cached)
  const uint32_t ob = (uint32_t)tb * c.row_bytes + c.lane_off, o0 = (uint32_t)t0 * c.row_bytes + c.lane_off;
  L.kb = ldg16(c.Ksc, ob);
  L.k0 = ldg16(c.Ksc, o0);
  if (WITH_V) {
    L.vb = ldg16(c.Vsc, ob);
    L.v0 = ldg16(c.Vsc, o0);
  }
  L.db = c.dseq ? c.dseq[tb] : 1;
  L.d0 = c.dseq ? c.dseq[t0] : 1;
  return L;
}

// returns the centroid's degree; *kp (and *vp) get the rounded pieces
template <bool WITH_V>
__device__ __forceinline__ int centroid_finish(const Ctx& c, const CentroidLoad<WITH_V>& L, uint4* kp, uint4* vp) {
  if (L.nm == 0) {
    *kp = L.kb;
    if (WITH_V) *vp = L.vb;
    return L.db;
  }
  float ak[8] = {0, 0, 0, 0, 0, 0, 0, 0}, av[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  fma_bf16x8(ak, L.kb, L.db);
  fma_bf16x8(ak, L.k0, L.d0);
  if (WITH_V) {
    fma_bf16x8(av, L.vb, L.db);
    fma_bf16x8(av, L.v0, L.d0);
  }
  int n = L.db + L.d0;
  for (int q = 1; q < L.nm; ++q) {
    const int tq = member_token(L.ip, c.mem0[L.st + q]);
    const uint32_t oq = (uint32_t)tq * c.row_bytes + c.lane_off;
    const int dq = c.dseq ? c.dseq[tq] : 1;
    fma_bf16x8(ak, ldg16(c.Ksc, oq), dq);
    if (WITH_V) fma_bf16x8(av, ldg16(c.Vsc, oq), dq);
    n += dq;
  }
  *kp = round_div_pack_bf16(ak, n);
  if (WITH_V) *vp = round_div_pack_bf16(av, n);
  return n;
}

__global__ __launch_bounds__(kThreads, 2) void fused2_kernel(
    const __bf16* __restrict__ K, const __bf16* __restrict__ V, const int32_t* __restrict__ deg_in,
    TensorView in, int seq, int n_super, float r1, __bf16* __restrict__ K_out, __bf16* __restrict__ V_out,
    int32_t* __restrict__ deg_out, TensorView out, int64_t deg_out_stride, int32_t* __restrict__ map_out) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* R = smem + kOffR;
  float* invb = reinterpret_cast<float*>(smem + kOffInvB);
  int16_t* dst0 = reinterpret_cast<int16_t*>(smem + kOffDst0);
  int32_t* cnt0 = reinterpret_cast<int32_t*>(smem + kOffCnt0);
  int16_t* start0 = reinterpret_cast<int16_t*>(smem + kOffStart0);
  int16_t* mem0 = reinterpret_cast<int16_t*>(smem + kOffMem0);
  float* inva_s = reinterpret_cast<float*>(smem + kOffInvA);
  int16_t* dst1 = reinterpret_cast<int16_t*>(smem + kOffDst1);
  float* score1 = reinterpret_cast<float*>(smem + kOffScore1);
  int* s_wave = reinterpret_cast<int*>(smem + kOffWave);
  int32_t* fill0 = reinterpret_cast<int32_t*>(smem + kOffFill0);
  int32_t* cnt1 = reinterpret_cast<int32_t*>(smem + kOffCnt1);
  int32_t* fill1 = reinterpret_cast<int32_t*>(smem + kOffFill1);
  int16_t* start1 = reinterpret_cast<int16_t*>(smem + kOffStart1);
  int16_t* mem1 = reinterpret_cast<int16_t*>(smem + kOffMem1);
  int16_t* lout1 = reinterpret_cast<int16_t*>(smem + kOffLout1);
  int16_t* srco1 = reinterpret_cast<int16_t*>(smem + kOffSrco1);

  const int sc = blockIdx.x % n_super, bh = blockIdx.x / n_super;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, col = lane & 31;
  const int piece = tid & (kOct - 1), r0 = tid >> 4;           // staging: row r0 + 32*it, 16-byte piece
  const int64_t tok0 = (int64_t)sc * 2 * kC;                    // first token of the super-chunk
  const __bf16* Ksc = K + in.seq_base(bh) + tok0 * in.stride_s;
  const __bf16* Vsc = V + in.seq_base(bh) + tok0 * in.stride_s;
  const int32_t* dsc = deg_in ? deg_in + (int64_t)bh * seq + tok0 : nullptr;

  int boff[kKSteps];            // this lane's fragment offsets inside a 32-row tile of R
#pragma unroll
  for (int s = 0; s < kKSteps; ++s) boff[s] = swz(col, 2 * s + half);
  const float* ib_lane = invb + 4 * half;

  bf16x8 afrag[2][kKSteps];
  float best[2];
  int bestj[2];
  // all 16 tiles of the 512 rows in R against this wave's 64 A rows; tiles are visited starting at
  // the wave's own neighbourhood so the running maxima settle early
  auto match_resident = [&]() {
    best[0] = best[1] = -INFINITY;
    bestj[0] = bestj[1] = 0;
    for (int k = 0; k < kH / 32; ++k) {
      const int ct = (2 * wave + k) & (kH / 32 - 1);
      const unsigned char* pb = R + ct * 32 * kRowB;
      f32x16 acc0 = {0}, acc1 = {0};
#pragma unroll
      for (int s = 0; s < kKSteps; ++s) {
        const bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(pb + boff[s]);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag, afrag[0][s], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag, afrag[1][s], acc1, 0, 0, 0);
      }
      f32x4 ib[4];
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) ib[qd] = *reinterpret_cast<const f32x4*>(ib_lane + ct * 32 + 8 * qd);
      tile_argmax<false>(acc0, ib, ct * 32, half, 32, best[0], bestj[0]);
      tile_argmax<false>(acc1, ib, ct * 32, half, 32, best[1], bestj[1]);
    }
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {   // the two lane halves of a row hold disjoint B rows
      const float ob = __shfl_xor(best[rt], 32);
      const int oj = __shfl_xor(bestj[rt], 32);
      if (ob > best[rt] || (ob == best[rt] && oj < bestj[rt])) { best[rt] = ob; bestj[rt] = oj; }
    }
  };

  // ---- M0: round-0 matching of the two chunks ---------------------------------------------------
  for (int x = 0; x < 2; ++x) {
    const __bf16* Kc = Ksc + (int64_t)x * kC * in.stride_s + piece * 8;
    {
      Piece xa[kH / 32];
#pragma unroll
      for (int it = 0; it < kH / 32; ++it)
        xa[it].u = *reinterpret_cast<const uint4*>(Kc + (int64_t)(2 * (r0 + 32 * it)) * in.stride_s);
#pragma unroll
      for (int it = 0; it < kH / 32; ++it) *reinterpret_cast<uint4*>(R + swz(r0 + 32 * it, piece)) = xa[it].u;
    }
    __syncthreads();
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      const int row = wave * 64 + rt * 32 + col;
#pragma unroll
      for (int s = 0; s < kKSteps; ++s)
        afrag[rt][s] = *reinterpret_cast<const bf16x8*>(R + swz(row, 2 * s + half));
    }
    __syncthreads();
    {
      Piece xb[kH / 32];
#pragma unroll
      for (int it = 0; it < kH / 32; ++it)
        xb[it].u = *reinterpret_cast<const uint4*>(Kc + (int64_t)(2 * (r0 + 32 * it) + 1) * in.stride_s);
#pragma unroll
      for (int it = 0; it < kH / 32; ++it) {
        const float ss = row_sum<kOct>(sumsq8(xb[it]));
        *reinterpret_cast<uint4*>(R + swz(r0 + 32 * it, piece)) = xb[it].u;
        if (piece == 0) invb[r0 + 32 * it] = inv_norm(ss);
      }
    }
    __syncthreads();
    match_resident();
    if (half == 0) {
      dst0[x * kH + wave * 64 + col] = (int16_t)bestj[0];
      dst0[x * kH + wave * 64 + 32 + col] = (int16_t)bestj[1];
    }
    __syncthreads();
  }

  // ---- B0: member lists of the round-0 centroids (r = 1: every source is merged) --------------
  cnt0[tid] = 0;
  cnt0[tid + kThreads] = 0;
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int s = tid + e * kThreads;                      // source s: chunk s>>9, A index s&511
    atomicAdd(&cnt0[(s & ~(kH - 1)) + dst0[s]], 1);
  }
  __syncthreads();
  int longest;
  {
    const int c0 = cnt0[2 * tid], c1 = cnt0[2 * tid + 1];
    longest = max(c0, c1);
    const int base = block_exclusive_scan8(c0 + c1, s_wave);
    start0[2 * tid] = (int16_t)base;
    start0[2 * tid + 1] = (int16_t)(base + c0);
    fill0[2 * tid] = 0;
    fill0[2 * tid + 1] = 0;
  }
  const bool any_long0 = __syncthreads_or(longest > kSortMax);
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int s = tid + e * kThreads;
    const int ip = (s & ~(kH - 1)) + dst0[s];
    int pos;
    if (any_long0 && cnt0[ip] > kSortMax) {
      pos = 0;
      for (int o = (s & ~(kH - 1)); o < s; ++o) pos += (dst0[o] == dst0[s]);
    } else {
      pos = atomicAdd(&fill0[ip], 1);
    }
    mem0[start0[ip] + pos] = (int16_t)(s & (kH - 1));
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int ip = 2 * tid + e;
    const int n = cnt0[ip];
    if (n > 1 && n <= kSortMax) {
      int16_t* lst = &mem0[start0[ip]];
      for (int a = 1; a < n; ++a) {
        const int16_t v = lst[a];
        int b2 = a - 1;
        while (b2 >= 0 && lst[b2] > v) { lst[b2 + 1] = lst[b2]; --b2; }
        lst[b2 + 1] = v;
      }
    }
  }
  __syncthreads();

  Ctx ctx{Ksc, Vsc, dsc, (uint32_t)in.stride_s * 2u, (uint32_t)piece * 16u, cnt0, start0, mem0};

  // ---- G0: round-0 centroid keys, on chip ---------------------------------------------------------
  // One row per 16 lanes (coalesced gathers), 4 centroids in flight per row group.  First the
  // round-1 A rows (even centroids) go through R into the MFMA operand registers of the wave that
  // owns them, then the round-1 B rows (odd centroids) are left resident in R.
  float inva1[2];
#pragma unroll 1
  for (int parity = 0; parity < 2; ++parity) {
    float* norms = parity == 0 ? inva_s : invb;
    for (int it = 0; it < kH / 32; it += 4) {
      CentroidLoad<false> ld[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) ld[u] = centroid_issue<false>(ctx, 2 * (r0 + 32 * (it + u)) + parity);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int row = r0 + 32 * (it + u);
        Piece pk;
        (void)centroid_finish<false>(ctx, ld[u], &pk.u, nullptr);
        const float ss = row_sum<kOct>(sumsq8(pk));
        *reinterpret_cast<uint4*>(R + swz(row, piece)) = pk.u;
        if (piece == 0) norms[row] = inv_norm(ss);
      }
    }
    __syncthreads();
    if (parity == 0) {
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) {
        const int row = wave * 64 + rt * 32 + col;
#pragma unroll
        for (int s = 0; s < kKSteps; ++s)
          afrag[rt][s] = *reinterpret_cast<const bf16x8*>(R + swz(row, 2 * s + half));
      }
      inva1[0] = inv_norm_of_operand_row<kKSteps>(afrag[0]);
      inva1[1] = inv_norm_of_operand_row<kKSteps>(afrag[1]);
      __syncthreads();
    }
  }

  // ---- M1: round-1 matching, everything on chip --------------------------------------------------
  match_resident();
  if (half == 0) {
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      const int i2 = wave * 64 + rt * 32 + col;
      dst1[i2] = (int16_t)bestj[rt];
      score1[i2] = best[rt] * inva1[rt];
    }
  }
  __syncthreads();   // R is free from here on

  // ---- B1: top-r of round 1, member lists, compaction --------------------------------------------
  const int m1 = merge_count(r1, kH);
  const int n_out = 2 * kH - m1;
  if (m1 < kH) {
    bool drop = true;
    if (m1 > 0) {
      const float si = score1[tid];
      int rank = 0;
      for (int o4 = 0; o4 < kH; o4 += 4) {
        const float4 so = *reinterpret_cast<const float4*>(&score1[o4]);
        rank += (so.x > si) || (so.x == si && o4 < tid);
        rank += (so.y > si) || (so.y == si && o4 + 1 < tid);
        rank += (so.z > si) || (so.z == si && o4 + 2 < tid);
        rank += (so.w > si) || (so.w == si && o4 + 3 < tid);
      }
      drop = rank >= m1;
    }
    if (drop) dst1[tid] = -1;
  }
  cnt1[tid] = 0;
  __syncthreads();
  const int d1 = dst1[tid];                                // this thread's round-1 source: A' index tid
  if (d1 >= 0) atomicAdd(&cnt1[d1], 1);
  __syncthreads();
  {
    const int c = cnt1[tid];
    const int base = block_exclusive_scan8(c, s_wave);
    start1[tid] = (int16_t)base;
    fill1[tid] = 0;
    longest = c;
  }
  const bool any_long1 = __syncthreads_or(longest > kSortMax);
  if (d1 >= 0) {
    int pos;
    if (any_long1 && cnt1[d1] > kSortMax) {
      pos = 0;
      for (int o = 0; o < tid; ++o) pos += (dst1[o] == d1);
    } else {
      pos = atomicAdd(&fill1[d1], 1);
    }
    mem1[start1[d1] + pos] = (int16_t)tid;
  }
  __syncthreads();
  {
    const int n = cnt1[tid];
    if (n > 1 && n <= kSortMax) {
      int16_t* lst = &mem1[start1[tid]];
      for (int a = 1; a < n; ++a) {
        const int16_t v = lst[a];
        int b2 = a - 1;
        while (b2 >= 0 && lst[b2] > v) { lst[b2 + 1] = lst[b2]; --b2; }
        lst[b2 + 1] = v;
      }
    }
  }
  {
    // centroids 2*tid (A', retained unless merged) and 2*tid+1 (B', always retained)
    const bool keepA = d1 < 0;
    int base = block_exclusive_scan8((int)keepA + 1, s_wave);
    if (keepA) { lout1[2 * tid] = (int16_t)base; srco1[base] = (int16_t)(2 * tid); ++base; }
    lout1[2 * tid + 1] = (int16_t)base;
    srco1[base] = (int16_t)(2 * tid + 1);
  }
  __syncthreads();

  const int out_base = sc * n_out;
  if (map_out != nullptr) {   // input token -> output slot, through both rounds
    int32_t* mp = map_out + (int64_t)bh * seq + tok0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int t = tid + e * kThreads;
      const int x = t >> 10, u = t & (kC - 1);
      const int ip = x * kH + ((u & 1) ? (u >> 1) : (int)dst0[x * kH + (u >> 1)]);
      const int dk = (ip & 1) ? -1 : (int)dst1[ip >> 1];
      mp[t] = out_base + ((dk < 0) ? lout1[ip] : lout1[2 * dk + 1]);
    }
  }

  // ---- E: output rows from the original keys and values -------------------------------------------
  int32_t* dout = deg_out + (int64_t)bh * deg_out_stride + out_base;
  constexpr int NRG = kThreads / kOct;   // 32 row groups
  char* Kob = reinterpret_cast<char*>(K_out + out.seq_base(bh) + (int64_t)out_base * out.stride_s);
  char* Vob = reinterpret_cast<char*>(V_out + out.seq_base(bh) + (int64_t)out_base * out.stride_s);
  const uint32_t orow = (uint32_t)out.stride_s * 2u;
  for (int ob = 0; ob < n_out; ob += 2 * NRG) {
    // two output rows per row group; for each the loads of its own centroid and of its first
    // round-1 source (keys and values, each with its first round-0 source) are started up front
    CentroidLoad<true> ld[2][2];
    int ip0[2], nm1[2], st1[2];
    bool valid[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int o = ob + u * NRG + r0;
      valid[u] = o < n_out;
      ip0[u] = srco1[valid[u] ? o : n_out - 1];
      nm1[u] = (ip0[u] & 1) ? cnt1[ip0[u] >> 1] : 0;
      st1[u] = (ip0[u] & 1) ? (int)start1[ip0[u] >> 1] : 0;
      const int ipm = nm1[u] > 0 ? 2 * (int)mem1[st1[u]] : ip0[u];
      ld[u][0] = centroid_issue<true>(ctx, ip0[u]);
      ld[u][1] = centroid_issue<true>(ctx, ipm);
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (!valid[u]) continue;
      const int o = ob + u * NRG + r0;
      const uint32_t oo = (uint32_t)o * orow + ctx.lane_off;
      uint4 k0, v0;
      const int n0 = centroid_finish<true>(ctx, ld[u][0], &k0, &v0);
      if (nm1[u] == 0) {
        stg16(Kob, oo, k0);
        stg16(Vob, oo, v0);
        if (piece == 0) dout[o] = n0;
        continue;
      }
      float ak[8] = {0, 0, 0, 0, 0, 0, 0, 0}, av[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      fma_bf16x8(ak, k0, n0);
      fma_bf16x8(av, v0, n0);
      int ntot = n0;
      {
        uint4 kq, vq;
        const int nq = centroid_finish<true>(ctx, ld[u][1], &kq, &vq);
        fma_bf16x8(ak, kq, nq);
        fma_bf16x8(av, vq, nq);
        ntot += nq;
      }
      for (int q = 1; q < nm1[u]; ++q) {
        const CentroidLoad<true> lq = centroid_issue<true>(ctx, 2 * (int)mem1[st1[u] + q]);
        uint4 kq, vq;
        const int nq = centroid_finish<true>(ctx, lq, &kq, &vq);
        fma_bf16x8(ak, kq, nq);
        fma_bf16x8(av, vq, nq);
        ntot += nq;
      }
      stg16(Kob, oo, round_div_pack_bf16(ak, ntot));
      stg16(Vob, oo, round_div_pack_bf16(av, ntot));
      if (piece == 0) dout[o] = ntot;
    }
  }
}

}  // namespace

bool fused2_supported(int dtype, int dim, int chunk, int seq, float r0) {
  return dtype == CKV_BF16 && dim == kD && chunk == kC && seq % (2 * kC) == 0 && r0 == 1.0f;
}

hipError_t launch_fused2(const void* K, const void* V, const int32_t* deg_in, TensorView in, int n_bh, int seq,
                         float r1, void* K_out, void* V_out, int32_t* deg_out, TensorView out,
                         int64_t deg_out_stride, int32_t* map_out, hipStream_t st) {
  static KernelSetup setup;
  if (hipError_t e = kernel_setup(reinterpret_cast<const void*>(&fused2_kernel), kLdsBytes, setup); e != hipSuccess) return e;
  const int n_super = seq / (2 * kC);
  const int64_t total = (int64_t)n_bh * n_super;
  // rows of a super-chunk are addressed with 32-bit byte offsets
  if (total > (1 << 30) || in.stride_s > (1 << 18) || out.stride_s > (1 << 18)) return hipErrorInvalidValue;
  ScopedTimer t("fused2_bf16", st);
  hipLaunchKernelGGL(fused2_kernel, dim3((int)total), dim3(kThreads), kLdsBytes, st,
                     static_cast<const __bf16*>(K), static_cast<const __bf16*>(V), deg_in, in, seq, n_super, r1,
                     static_cast<__bf16*>(K_out), static_cast<__bf16*>(V_out), deg_out, out, deg_out_stride,
                     map_out);
  return hipGetLastError();
}

}  // namespace ckv
