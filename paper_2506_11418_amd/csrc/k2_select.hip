// Top-r over ALL chunks of a sequence: the reading of Sec. 5.2-5.3 in which the candidate edges of
// every chunk of a sequence enter one common ranking and the best fraction r of them is merged.
//
// One workgroup per (batch, head) sequence finds the cut of the ranking (score descending, position
// ascending) below its m = floor(r * edges) best edges with a 4-pass radix select over the fp32
// scores, then counts for every chunk how many of its edges lie above the cut and prefix-sums the
// chunks' output offsets.  The merge kernel then keeps, in each chunk, that many of the chunk's
// best edges under the same order, which is exactly the part of the global top-m that falls into
// the chunk.  Everything is integer work on the stored scores: the result is deterministic.
#include "ckv_internal.h"

namespace ckv {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

// fp32 -> uint32 whose unsigned order is the float order (-0 and +0 compare equal, as they do
// in the merge kernel's float comparisons)
__device__ inline uint32_t order_key(float x) {
  const uint32_t u = __float_as_uint(x + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ inline int block_scan_excl(int v, int* s_wave, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(inc, d);
    if (lane >= d) inc += o;
  }
  if (lane == 63) s_wave[wave] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const int t = s_wave[w];
    if (w < wave) base += t;
    tot += t;
  }
  __syncthreads();
  *total = tot;
  return base + inc - v;
}

// table[bh * n_chunks + g] = (edges of chunk g that are merged, first output row of chunk g)
__global__ __launch_bounds__(kSelThreads) void global_select_kernel(const float* __restrict__ score, int seq,
                                                                    int chunk, int n_chunks, float r,
                                                                    int2* __restrict__ table) {
  __shared__ int s_hist[256];
  __shared__ int s_wave[kSelWaves];
  __shared__ uint32_t s_prefix;
  __shared__ int s_k;

  const int bh = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_src = n_sources(seq, chunk);
  const int half = chunk >> 1;
  const int tail = seq % chunk;
  const int n_edges = n_src - (tail == 1 ? 1 : 0);      // a one-token tail chunk has no B token
  const int m = merge_count(r, n_edges);
  const float* sc = score + (int64_t)bh * n_src;
  int2* tab = table + (int64_t)bh * n_chunks;

  uint32_t cut = 0;      // key of the m-th best edge
  int quota = 0;         // edges with key == cut that are merged (the lowest positions)
  const bool all = (m >= n_edges), none = (m == 0);
  if (!all && !none) {
    if (tid == 0) { s_prefix = 0; s_k = m; }
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      if (tid < 256) s_hist[tid] = 0;
      __syncthreads();
      const uint32_t prefix = s_prefix;
      const uint32_t mask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
      for (int i = tid; i < n_edges; i += kSelThreads) {
        const uint32_t k = order_key(sc[i]);
        if ((k & mask) == prefix) atomicAdd(&s_hist[(k >> shift) & 255], 1);
      }
      __syncthreads();
      if (tid == 0) {   // walk the digits from the top until the wanted rank falls into one
        int k = s_k, d = 255;
        for (; d > 0; --d) {
          const int c = s_hist[d];
          if (c >= k) break;
          k -= c;
        }
        s_k = k;
        s_prefix = prefix | ((uint32_t)d << shift);
      }
      __syncthreads();
    }
    cut = s_prefix;
    quota = s_k;
  }

  // ---- per chunk: edges above the cut and edges on it -----------------------------------------
  // table is used as scratch first: (.x = above, .y = on the cut)
  if (half >= 32) {      // a wave per chunk
    for (int g = wave; g < n_chunks; g += kSelWaves) {
      const int L = min(chunk, seq - g * chunk);
      const int nA = (L >= 2) ? (L + 1) >> 1 : 0;
      int gt = 0, eq = 0;
      if (all) gt = nA;
      else if (!none)
        for (int i0 = 0; i0 < nA; i0 += 64) {
          const int i = i0 + lane;
          const uint32_t k = (i < nA) ? order_key(sc[g * half + i]) : 0u;
          gt += __popcll(__ballot(i < nA && k > cut));
          eq += __popcll(__ballot(i < nA && k == cut));
        }
      if (lane == 0) tab[g] = make_int2(gt, eq);
    }
  } else {               // a thread per chunk
    for (int g = tid; g < n_chunks; g += kSelThreads) {
      const int L = min(chunk, seq - g * chunk);
      const int nA = (L >= 2) ? (L + 1) >> 1 : 0;
      int gt = 0, eq = 0;
      if (all) gt = nA;
      else if (!none)
        for (int i = 0; i < nA; ++i) {
          const uint32_t k = order_key(sc[g * half + i]);
          gt += (k > cut);
          eq += (k == cut);
        }
      tab[g] = make_int2(gt, eq);
    }
  }
  __syncthreads();

  // ---- chunks in order: hand the quota of on-the-cut edges to the earliest ones, offsets ------
  int eq_before = 0, out_before = 0;
  for (int g0 = 0; g0 < n_chunks; g0 += kSelThreads) {
    const int g = g0 + tid;
    int2 c = make_int2(0, 0);
    int L = 0;
    if (g < n_chunks) { c = tab[g]; L = min(chunk, seq - g * chunk); }
    int tot_eq, tot_out;
    const int eq_excl = eq_before + block_scan_excl(c.y, s_wave, &tot_eq);
    const int take = max(0, min(c.y, quota - eq_excl));
    const int kept = c.x + take;
    const int out_excl = out_before + block_scan_excl(L - kept, s_wave, &tot_out);
    if (g < n_chunks) tab[g] = make_int2(kept, out_excl);
    eq_before += tot_eq;
    out_before += tot_out;
  }
}

}  // namespace

hipError_t launch_global_select(const float* score, int n_bh, int seq, int chunk, float r, int32_t* table,
                                hipStream_t st) {
  ScopedTimer t("global_select", st);
  hipLaunchKernelGGL(global_select_kernel, dim3(n_bh), dim3(kSelThreads), 0, st, score, seq, chunk,
                     div_up(seq, chunk), r, reinterpret_cast<int2*>(table));
  return hipGetLastError();
}

}  // namespace ckv
