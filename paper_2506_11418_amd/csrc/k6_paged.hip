// Block-paged KV caches (the layout of a serving engine's block manager): moving a sequence's tokens
// between a block pool and the strided tensors the clustering kernels work on, and releasing the
// blocks a compressed sequence no longer needs.  Pure data movement: 16-byte pieces, one table
// lookup per row.
#include "ckv_internal.h"
#include "ckv_device.h"

namespace ckv {
namespace {

// one thread per 16-byte piece of one (batch, head, token) row
template <bool TO_POOL>
__global__ void paged_move_kernel(unsigned char* __restrict__ K_pool, unsigned char* __restrict__ V_pool,
                                  int32_t* __restrict__ deg_pool, const int32_t* __restrict__ table, int max_blocks,
                                  int shift, int n_blocks, int heads, int seq, int pieces_per_row,
                                  unsigned char* __restrict__ K, unsigned char* __restrict__ V,
                                  int32_t* __restrict__ deg, TensorView view, int elem_bytes, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  // piece fastest, then token, then head: consecutive threads walk one head's tokens, which are
  // contiguous in the tensor and, block by block, in the pool
  const int piece = (int)(e % pieces_per_row);
  int64_t x = e / pieces_per_row;
  const int t = (int)(x % seq);
  x /= seq;
  const int h = (int)(x % heads), b = (int)(x / heads);
  const int blk = table[(int64_t)b * max_blocks + (t >> shift)];
  const bool in_pool = (unsigned)blk < (unsigned)n_blocks;
  // pool: [n_blocks, heads, block_size, dim]
  const int64_t row = in_pool ? ((((int64_t)blk * heads + h) << shift) + (t & ((1 << shift) - 1))) : 0;
  const int64_t poff = (row * pieces_per_row + piece) * 16;
  const int64_t toff = ((int64_t)b * view.stride_b + (int64_t)h * view.stride_h + (int64_t)t * view.stride_s) *
                           elem_bytes + piece * 16;
  const int64_t doff = ((int64_t)b * heads + h) * view.deg_stride + t;
  if (TO_POOL) {
    if (!in_pool) return;
    if (K) stg16_stream(K_pool + poff, *reinterpret_cast<const uint4*>(K + toff));
    if (V) stg16_stream(V_pool + poff, *reinterpret_cast<const uint4*>(V + toff));
    if (piece == 0 && deg_pool && (deg || K)) deg_pool[row] = deg ? deg[doff] : 1;
  } else {
    const uint4 zero = make_uint4(0, 0, 0, 0);
    *reinterpret_cast<uint4*>(K + toff) = in_pool ? ldg16_stream(K_pool + poff) : zero;
    *reinterpret_cast<uint4*>(V + toff) = in_pool ? ldg16_stream(V_pool + poff) : zero;
    if (piece == 0 && deg) deg[doff] = (in_pool && deg_pool) ? deg_pool[row] : 1;
  }
}

// Decode-step cache update on pages: the new token of sequence b goes to position lens[b] of every
// head (degree 1).  A sequence whose next position has no valid block is left alone.  One workgroup
// per sequence, which also advances lens[b] once all of its threads have read it.
__global__ void paged_append_kernel(const unsigned char* __restrict__ k_new, const unsigned char* __restrict__ v_new,
                                    unsigned char* __restrict__ K_pool, unsigned char* __restrict__ V_pool,
                                    int32_t* __restrict__ deg_pool, const int32_t* __restrict__ table, int max_blocks,
                                    int shift, int n_blocks, int heads, int32_t* __restrict__ lens,
                                    int pieces_per_row) {
  const int b = blockIdx.x;
  const int t = lens[b];
  __syncthreads();
  if (t < 0 || (t >> shift) >= max_blocks) return;       // the same for every thread of the workgroup
  const int blk = table[(int64_t)b * max_blocks + (t >> shift)];
  if ((unsigned)blk >= (unsigned)n_blocks) return;
  const int per_seq = heads * pieces_per_row;
  for (int e = threadIdx.x; e < per_seq; e += blockDim.x) {
    const int piece = e % pieces_per_row, h = e / pieces_per_row;
    const int64_t row = (((int64_t)blk * heads + h) << shift) + (t & ((1 << shift) - 1));
    const int64_t so = (((int64_t)b * heads + h) * pieces_per_row + piece) * 16;
    const int64_t poff = (row * pieces_per_row + piece) * 16;
    *reinterpret_cast<uint4*>(K_pool + poff) = *reinterpret_cast<const uint4*>(k_new + so);
    *reinterpret_cast<uint4*>(V_pool + poff) = *reinterpret_cast<const uint4*>(v_new + so);
    if (piece == 0 && deg_pool) deg_pool[row] = 1;
  }
  if (threadIdx.x == 0) lens[b] = t + 1;
}

__global__ void paged_release_kernel(int32_t* __restrict__ table, int max_blocks, int n_b, int keep_blocks,
                                     int old_blocks, int32_t* __restrict__ freed, int freed_stride,
                                     int32_t* __restrict__ lens, int seq) {
  const int n_freed = old_blocks - keep_blocks;
  const int width = freed_stride > n_freed ? freed_stride : n_freed;   // per sequence: released entries, then padding
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (width > 0 && e < n_b * width) {
    const int b = e / width, k = e % width;
    if (k < n_freed) {
      int32_t* slot = table + (int64_t)b * max_blocks + keep_blocks + k;
      if (freed) freed[(int64_t)b * freed_stride + k] = *slot;
      *slot = -1;
    } else if (freed) {
      freed[(int64_t)b * freed_stride + k] = -1;
    }
  }
  if (lens && e < n_b) lens[e] = seq;
}

}  // namespace

hipError_t launch_paged_gather(const void* K_pool, const void* V_pool, const int32_t* deg_pool, PagedView paged,
                               int n_b, int heads, int seq, int row_bytes, void* K, void* V, int32_t* deg,
                               TensorView out, int elem_bytes, hipStream_t st) {
  const int ppr = row_bytes / 16;
  const int64_t total = (int64_t)n_b * heads * seq * ppr;
  if (total == 0) return hipSuccess;
  ScopedTimer t("paged_gather", st);
  hipLaunchKernelGGL(paged_move_kernel<false>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     static_cast<unsigned char*>(const_cast<void*>(K_pool)),
                     static_cast<unsigned char*>(const_cast<void*>(V_pool)), const_cast<int32_t*>(deg_pool),
                     paged.table, paged.max_blocks, paged.shift, paged.n_blocks, heads, seq, ppr,
                     static_cast<unsigned char*>(K), static_cast<unsigned char*>(V), deg, out, elem_bytes, total);
  return hipGetLastError();
}

hipError_t launch_paged_append(const void* k_new, const void* v_new, void* K_pool, void* V_pool, int32_t* deg_pool,
                               PagedView paged, int n_b, int heads, int row_bytes, int32_t* lens, hipStream_t st) {
  const int ppr = row_bytes / 16;
  ScopedTimer t("paged_append", st);
  hipLaunchKernelGGL(paged_append_kernel, dim3((unsigned)n_b), dim3(256), 0, st,
                     static_cast<const unsigned char*>(k_new), static_cast<const unsigned char*>(v_new),
                     static_cast<unsigned char*>(K_pool), static_cast<unsigned char*>(V_pool), deg_pool, paged.table,
                     paged.max_blocks, paged.shift, paged.n_blocks, heads, lens, ppr);
  return hipGetLastError();
}

hipError_t launch_paged_scatter(const void* K, const void* V, const int32_t* deg, TensorView in, int n_b, int heads,
                                int seq, int row_bytes, int elem_bytes, void* K_pool, void* V_pool,
                                int32_t* deg_pool, int32_t* table, int max_blocks, int shift, int n_blocks,
                                int keep_blocks, int old_blocks, int32_t* freed, int freed_stride, int32_t* lens,
                                hipStream_t st) {
  const int ppr = row_bytes / 16;
  const int64_t total = (int64_t)n_b * heads * seq * ppr;
  if (total > 0 && (K || V || deg)) {
    ScopedTimer t("paged_scatter", st);
    hipLaunchKernelGGL(paged_move_kernel<true>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       static_cast<unsigned char*>(K_pool), static_cast<unsigned char*>(V_pool), deg_pool, table,
                       max_blocks, shift, n_blocks, heads, seq, ppr,
                       static_cast<unsigned char*>(const_cast<void*>(K)),
                       static_cast<unsigned char*>(const_cast<void*>(V)), const_cast<int32_t*>(deg), in, elem_bytes,
                       total);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int n_freed = old_blocks - keep_blocks;
  const int width = (freed && freed_stride > n_freed) ? freed_stride : n_freed;
  const int work = n_b * width;
  const int n = work > n_b ? work : n_b;
  if (n <= 0) return hipSuccess;
  ScopedTimer t("paged_release", st);
  hipLaunchKernelGGL(paged_release_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, table, max_blocks,
                     n_b, keep_blocks, old_blocks, freed, freed ? freed_stride : 0, lens, seq);
  return hipGetLastError();
}

}  // namespace ckv
