// Internal declarations shared by the host driver and the kernel translation units of libckv.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "ckv.h"

namespace ckv {

// Strides (in elements) of one [batch*heads] x seq x dim tensor as the kernels see it.
struct TensorView {
  int64_t stride_b, stride_h, stride_s;
  int32_t heads;  // to split a flat (batch*heads) index
  int64_t deg_stride;  // elements between the degree rows of consecutive (batch, head) sequences
  __host__ __device__ inline int64_t seq_base(int bh) const {
    return (int64_t)(bh / heads) * stride_b + (int64_t)(bh % heads) * stride_h;
  }
};

// A block-paged cache: token t of sequence b lives in block table[b*max_blocks + (t >> shift)] at
// offset t & ((1 << shift) - 1).  table == nullptr: not paged.
struct PagedView {
  const int32_t* table;
  int32_t max_blocks, shift, n_blocks;
};

// One side (the input rows, the output rows, ...) of a launch that lives in a block pool instead of
// a strided tensor: token t of the launch's view is token tok0 + t of the sequence, and token u of
// sequence b, head h is pool row ((table[b*max_blocks + (u >> shift)] * heads + h) << shift) +
// (u & (block_size - 1)) of a [n_blocks, heads, block_size, dim] pool (degrees: the same row of a
// [n_blocks, heads, block_size] pool).  table == nullptr: the side is a strided tensor.
struct PagedSide {
  const int32_t* table = nullptr;
  int32_t max_blocks = 0, shift = 0, n_blocks = 0, tok0 = 0;
};

inline __host__ __device__ int div_up(int a, int b) { return (a + b - 1) / b; }

// Number of A tokens (sources) in a sequence of `seq` tokens cut into chunks of `chunk` (even).
inline __host__ __device__ int n_sources(int seq, int chunk) {
  int full = seq / chunk, tail = seq % chunk;
  return full * (chunk / 2) + (tail + 1) / 2;
}

// floor(r * n_a + 1e-9) with r widened from float: edges merged in a chunk with n_a sources.
inline __host__ __device__ int merge_count(float r, int n_a) {
  return (int)((double)r * (double)n_a + 1e-9);
}

// Tokens a chunk of L tokens keeps after one round with merge fraction r.
inline __host__ __device__ int chunk_out(int L, float r) {
  return (L < 2) ? L : L - merge_count(r, (L + 1) / 2);
}

// ---- kernel launchers (each returns hipGetLastError() after the launch) ------------------------
// Similarity + per-source argmax.  dst_local[bh, i] = index within the chunk's B set, score fp32.
hipError_t launch_match(const void* K, int dtype, int dim, TensorView kv, int n_bh, int seq,
                        int chunk, int32_t* dst_local, float* score, hipStream_t st, PagedSide paged = PagedSide{});

// Turn chunk-local B indices into sequence positions (for ckv_match's public output).
hipError_t launch_dst_positions(const int32_t* dst_local, int32_t* dst_pos, int n_bh, int seq,
                                int chunk, hipStream_t st);

// Two consecutive rounds whose first merges every edge (r = 1) can skip the intermediate VALUE
// cache.  The first round's merge then writes keys and degrees only and exports every chunk's
// member lists (lists_out: per (sequence, chunk) 3*(chunk/2) int16: count | start | members); the
// second round's merge rebuilds each value row of its input from the original values through
// those lists (same arithmetic, same single rounding: bit-identical results).
struct ValueOrigin {
  const void* V0;         // the first round's value input, at the first clustered token
  TensorView view0;       // its layout (deg_stride: row stride of deg0)
  const int32_t* deg0;    // the first round's degree input at the first clustered token, or NULL (= 1)
  const int16_t* lists;   // what the first round's merge exported
  int32_t seq0;           // tokens the first round clustered
  int32_t n_chunks0;      // its chunks per sequence
  PagedSide paged;        // V0 / deg0 are block pools (then V0, deg0 point at the pools, view0.heads = heads)
};

// Per-chunk top-r selection + degree-weighted merge + order-preserving compaction.
// map_out[bh*map_stride + t] (t < seq) = map_offset + output index of the centroid input token t
// joined; may be NULL.  deg_in[bh*deg_in_stride + t].  lists_out != NULL: keys-only first round of a
// deferred-value pair (V, V_out unused); org != NULL: its second round (V unused).
hipError_t launch_merge(const void* K, const void* V, const int32_t* deg_in, int dtype, int dim,
                        TensorView in, int n_bh, int seq, int chunk, float r,
                        const int32_t* dst_local, const float* score, void* K_out, void* V_out,
                        int32_t* deg_out, TensorView out, int64_t deg_out_stride, int32_t* map_out,
                        int64_t deg_in_stride, int64_t map_stride, int map_offset, const int32_t* sel_table,
                        int16_t* lists_out, const ValueOrigin* org, hipStream_t st, PagedSide paged_in = PagedSide{},
                        PagedSide paged_out_k = PagedSide{}, PagedSide paged_out_v = PagedSide{});

// Selection over all chunks of a sequence: from the match scores, table[bh, chunk] = (edges of the
// chunk among the sequence's floor(r * edges) best, first output row of the chunk), two int32 each.
// launch_merge with sel_table = table then merges exactly those.
hipError_t launch_global_select(const float* score, int n_bh, int seq, int chunk, float r, int32_t* table,
                                hipStream_t st);

// Decode-step cache update: row lens[b] (device, then incremented) or `pos` of every (batch, head)
// := (k_new, v_new, degree 1).  k_new, v_new: [batch, heads, dim] contiguous.
hipError_t launch_append(const void* k_new, const void* v_new, void* K, void* V, int32_t* deg, TensorView cache,
                         int batch, int capacity, int32_t* lens, int pos, int row_bytes, int elem_bytes,
                         hipStream_t st);

// Copy the first n_head and the last n_tail tokens of every sequence (sinks / recents) to the
// head / tail of the output, with their degrees and their entries of the round's map.
hipError_t launch_edges(const void* K, const void* V, const int32_t* deg_in, TensorView in, int in_len, void* K_out,
                        void* V_out, int32_t* deg_out, TensorView out, int64_t deg_out_stride, int out_len,
                        int32_t* map_out, int n_head, int n_tail, int n_bh, int row_bytes, int elem_bytes,
                        hipStream_t st, PagedSide paged_in = PagedSide{}, PagedSide paged_out_k = PagedSide{},
                        PagedSide paged_out_v = PagedSide{});

// assign[bh, t] = map[bh, assign[bh, t]] for t < seq0.
hipError_t launch_compose(int32_t* assign, const int32_t* map, int n_bh, int seq0, int map_len,
                          hipStream_t st);

// Plain strided copy of [n_bh, seq, dim] rows (used when the schedule has zero rounds).
hipError_t launch_copy_rows(const void* src, TensorView in, void* dst, TensorView out, int n_bh,
                            int seq, int row_bytes, int elem_bytes, hipStream_t st);
hipError_t launch_fill_deg(const int32_t* deg_in, int64_t in_stride, int32_t* deg_out, int64_t out_stride, int32_t* assign,
                           int n_bh, int seq, hipStream_t st);

// Decode attention: split along the sequence; the slice that finishes last merges the partials.
// The workspace starts with attn_counter_bytes() of int32 arrival counters that are zero between calls
// (launch_decode_attn with counters != NULL keeps them there instead and uses the whole workspace for
// the partial results).
size_t attn_counter_bytes(int n_b, int kv_heads);
// span_limit > 0 (paged caches): no slice may cover more tokens than that
int attn_splits(int n_b, int kv_heads, int seq, int span_limit);
int attn_paged_span_limit(int block_size);
size_t attn_workspace_bytes(int n_b, int kv_heads, int q_heads, int dim, int seq, int span_limit);
hipError_t launch_decode_attn(const void* q, int q_heads, const void* K, const void* V, int dtype,
                              int dim, TensorView kv, int n_b, int kv_heads, int seq,
                              const int32_t* lens, const int32_t* deg, float scale, void* o,
                              int o_dtype, void* workspace, PagedView paged, hipStream_t st,
                              int32_t* counters = nullptr);

// Block pool <-> strided tensors.  pool: [n_blocks, heads, block_size, dim] (deg pool
// [n_blocks, heads, block_size]); the first `seq` tokens of every sequence are moved.  Gather writes
// zeros (degree 1) for tokens whose table entry lies outside the pool; scatter skips them.
hipError_t launch_paged_gather(const void* K_pool, const void* V_pool, const int32_t* deg_pool, PagedView paged,
                               int n_b, int heads, int seq, int row_bytes, void* K, void* V, int32_t* deg,
                               TensorView out, int elem_bytes, hipStream_t st);
// Decode-step update of a paged cache: token lens[b] of every head := (k_new, v_new, degree 1), then
// lens[b] += 1; a sequence whose next position has no block inside the pool is left alone.
hipError_t launch_paged_append(const void* k_new, const void* v_new, void* K_pool, void* V_pool, int32_t* deg_pool,
                               PagedView paged, int n_b, int heads, int row_bytes, int32_t* lens, hipStream_t st);
// Scatter also releases blocks: entries [keep_blocks, old_blocks) of every table row are copied to
// freed[b*freed_stride + k] (if freed != NULL; the rest of a row is set to -1) and set to -1, and
// lens[b] := seq (if lens != NULL).  K, V or deg may be NULL: that tensor is then not moved.
hipError_t launch_paged_scatter(const void* K, const void* V, const int32_t* deg, TensorView in, int n_b, int heads,
                                int seq, int row_bytes, int elem_bytes, void* K_pool, void* V_pool,
                                int32_t* deg_pool, int32_t* table, int max_blocks, int shift, int n_blocks,
                                int keep_blocks, int old_blocks, int32_t* freed, int freed_stride, int32_t* lens,
                                hipStream_t st);

// ---- timing hooks ----------------------------------------------------------------------------
// One-time set-up of a kernel that needs more than the default dynamic LDS, per device (each device
// holds its own copy of the code object, so the limit is raised on each one that launches it).
// `state` is the call site's own table; first use on a device happens under its lock, later calls
// read one atomic flag.
constexpr int kMaxDevices = 64;
struct KernelSetup {
  std::mutex lock;
  std::atomic<bool> done[kMaxDevices];
  int n_cu[kMaxDevices];
  KernelSetup() {
    for (int i = 0; i < kMaxDevices; ++i) { done[i].store(false, std::memory_order_relaxed); n_cu[i] = 0; }
  }
};
inline hipError_t kernel_setup(const void* kernel, size_t dynamic_lds, KernelSetup& state, int* n_cu = nullptr) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!state.done[dev].load(std::memory_order_acquire)) {
    std::lock_guard<std::mutex> g(state.lock);
    if (!state.done[dev].load(std::memory_order_relaxed)) {
      int v = 0;
      e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev);
      if (e == hipSuccess)
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dynamic_lds);
      if (e != hipSuccess) return e;
      state.n_cu[dev] = v > 0 ? v : 256;
      state.done[dev].store(true, std::memory_order_release);
    }
  }
  if (n_cu) *n_cu = state.n_cu[dev];
  return hipSuccess;
}

bool timing_begin(const char* name, hipStream_t st);   // false: this launch is not being timed
void timing_end(hipStream_t st);
struct ScopedTimer {
  hipStream_t st;
  bool on;
  ScopedTimer(const char* name, hipStream_t s) : st(s), on(timing_begin(name, s)) {}
  ~ScopedTimer() { if (on) timing_end(st); }
};

}  // namespace ckv
