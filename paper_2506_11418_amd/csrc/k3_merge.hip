// Top-r selection, degree-weighted merge and order-preserving compaction of one clustering round
// (Sec. 5.3: "rank all candidate matches by similarity and only merge the top fraction"; the
// centroid equation; values merged with the same weights).
//
// One workgroup per (sequence, chunk).  Integer bookkeeping lives in LDS:
//   keep[i]      source i is among the m = floor(r*|A|) best edges (score desc, index asc);
//   members[]    kept sources grouped by destination, ascending inside a group (rank by counting:
//                no atomics decide an order, so results are run-to-run identical);
//   local_out[]  prefix sum over retained tokens (all B tokens, unkept A tokens).
// Rows are then produced gather-style: 16-byte pieces, one row per group of row_bytes/16 lanes,
// fp32 accumulation for bf16 (fp64 for fp32 storage), one rounding to the storage type.
#include "ckv_internal.h"

namespace ckv {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxHalf = 1024;  // max |A| = |B| (chunk <= 2048)

// Quotient S/n rounded to bf16 with a single nearest-even rounding: the fp32 quotient is
// correctly rounded, so a second rounding can only go wrong when it sits exactly on a bf16
// midpoint; the sign of the exact residual S - q*n then says on which side the true value lies.
__device__ inline uint16_t div_round_bf16(float S, float n) {
  const float q = S / n;
  const uint32_t u = __float_as_uint(q);
  const uint32_t low = u & 0xffffu;
  uint32_t up;
  if (low == 0x8000u) {
    const float res = fmaf(-q, n, S);
    up = (res == 0.f) ? ((u >> 16) & 1u) : (((res > 0.f) == (q > 0.f)) ? 1u : 0u);
  } else {
    up = low > 0x8000u;
  }
  return (uint16_t)((u >> 16) + up);
}

__device__ inline int block_exclusive_scan(int v, int* s_wave_tot, int* total) {
  // 256 threads = 4 waves
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(inc, d);
    if (lane >= d) inc += o;
  }
  if (lane == 63) s_wave_tot[wave] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const int t = s_wave_tot[w];
    if (w < wave) base += t;
    tot += t;
  }
  __syncthreads();
  *total = tot;
  return base + inc - v;
}

template <typename T>
struct Row;  // per-lane 16-byte piece arithmetic

template <>
struct Row<__bf16> {
  static constexpr int E = 8;
  typedef float Acc;
  __device__ static void load(const __bf16* p, float* x) {
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(w[i] << 16);
      x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ static void store_div(__bf16* p, const float* acc, int n) {
    uint32_t w[4];
    const float fn = (float)n;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      w[i] = (uint32_t)div_round_bf16(acc[2 * i], fn) | ((uint32_t)div_round_bf16(acc[2 * i + 1], fn) << 16);
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

template <>
struct Row<float> {
  static constexpr int E = 4;
  typedef double Acc;
  __device__ static void load(const float* p, float* x) {
    const float4 u = *reinterpret_cast<const float4*>(p);
    x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w;
  }
  __device__ static void store_div(float* p, const double* acc, int n) {
    const double dn = (double)n;
    *reinterpret_cast<float4*>(p) = make_float4((float)(acc[0] / dn), (float)(acc[1] / dn),
                                                (float)(acc[2] / dn), (float)(acc[3] / dn));
  }
};

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void merge_kernel(
    const T* __restrict__ K, const T* __restrict__ V, const int32_t* __restrict__ deg_in, TensorView in,
    int seq, int chunk, int n_chunks, float r, const int32_t* __restrict__ dst_local,
    const float* __restrict__ score, T* __restrict__ K_out, T* __restrict__ V_out,
    int32_t* __restrict__ deg_out, TensorView out, int64_t deg_out_stride, int32_t* __restrict__ map_out) {
  constexpr int E = Row<T>::E;
  constexpr int LPR = D / E;                 // lanes per row
  constexpr int NRG = kThreads / LPR;        // rows in flight per workgroup
  typedef typename Row<T>::Acc Acc;

  __shared__ int32_t s_dst[kMaxHalf];
  __shared__ float s_score[kMaxHalf];
  __shared__ unsigned char s_keep[kMaxHalf];
  __shared__ int32_t s_cnt[kMaxHalf];
  __shared__ int32_t s_start[kMaxHalf];
  __shared__ int16_t s_members[kMaxHalf];
  __shared__ int16_t s_local_out[2 * kMaxHalf];
  __shared__ int16_t s_src_of_out[2 * kMaxHalf];
  __shared__ int s_wave_tot[4];

  const int g = blockIdx.x % n_chunks, bh = blockIdx.x / n_chunks;
  const int tid = threadIdx.x;
  const int g0 = g * chunk, L = min(chunk, seq - g0);
  const int nA = (L + 1) >> 1, nB = L >> 1;
  const int m = (nB > 0) ? merge_count(r, nA) : 0;
  const int n_out = L - m;
  const int out_base = g * chunk_out(chunk, r);
  const int n_src = n_sources(seq, chunk);
  const int64_t src_base = (int64_t)bh * n_src + (int64_t)g * (chunk >> 1);

  for (int i = tid; i < nA; i += kThreads) {
    s_dst[i] = dst_local[src_base + i];
    s_score[i] = score[src_base + i];
  }
  for (int j = tid; j < nB; j += kThreads) s_cnt[j] = 0;
  __syncthreads();

  // ---- top-r: rank by counting ---------------------------------------------------------------
  if (m == nA || m == 0) {
    for (int i = tid; i < nA; i += kThreads) s_keep[i] = (m != 0);
  } else {
    for (int i = tid; i < nA; i += kThreads) {
      const float si = s_score[i];
      int rank = 0;
      for (int o = 0; o < nA; ++o) {
        const float so = s_score[o];
        rank += (so > si) || (so == si && o < i);
      }
      s_keep[i] = rank < m;
    }
  }
  __syncthreads();

  // ---- kept sources grouped by destination, ascending within a group --------------------------
  int my_pos[kMaxHalf / kThreads];
#pragma unroll
  for (int it = 0; it < kMaxHalf / kThreads; ++it) {
    const int i = tid + it * kThreads;
    my_pos[it] = 0;
    if (i < nA && s_keep[i]) {
      const int d = s_dst[i];
      int pos = 0;
      for (int o = 0; o < i; ++o) pos += (s_keep[o] && s_dst[o] == d);
      my_pos[it] = pos;
      atomicAdd(&s_cnt[d], 1);   // integer count: the total does not depend on the order
    }
  }
  __syncthreads();
  {
    int c[4], sum = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int j = tid * 4 + e;
      c[e] = (j < nB) ? s_cnt[j] : 0;
      sum += c[e];
    }
    int tot;
    int base = block_exclusive_scan(sum, s_wave_tot, &tot);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int j = tid * 4 + e;
      if (j < nB) s_start[j] = base;
      base += c[e];
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < kMaxHalf / kThreads; ++it) {
    const int i = tid + it * kThreads;
    if (i < nA && s_keep[i]) s_members[s_start[s_dst[i]] + my_pos[it]] = (int16_t)i;
  }

  // ---- retained tokens: prefix sum over the chunk --------------------------------------------
  {
    int flags = 0, cnt = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int u = tid * 8 + e;
      const bool ret = (u < L) && ((u & 1) || !s_keep[u >> 1]);
      flags |= (int)ret << e;
      cnt += ret;
    }
    int tot;
    int base = block_exclusive_scan(cnt, s_wave_tot, &tot);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int u = tid * 8 + e;
      if ((flags >> e) & 1) {
        s_local_out[u] = (int16_t)base;
        s_src_of_out[base] = (int16_t)u;
        ++base;
      }
    }
  }
  __syncthreads();

  // ---- assignment map of this round ----------------------------------------------------------
  if (map_out != nullptr) {
    int32_t* mp = map_out + (int64_t)bh * seq + g0;
    for (int u = tid; u < L; u += kThreads) {
      const bool ret = (u & 1) || !s_keep[u >> 1];
      const int slot = ret ? s_local_out[u] : s_local_out[2 * s_dst[u >> 1] + 1];
      mp[u] = out_base + slot;
    }
  }

  // ---- emit rows -----------------------------------------------------------------------------
  const int rg = tid / LPR, piece = tid % LPR;
  const int64_t in_seq = in.seq_base(bh) + (int64_t)g0 * in.stride_s + piece * E;
  const int64_t out_seq = out.seq_base(bh) + (int64_t)out_base * out.stride_s + piece * E;
  const int32_t* dseq = deg_in ? deg_in + (int64_t)bh * seq + g0 : nullptr;
  int32_t* dout = deg_out + (int64_t)bh * deg_out_stride + out_base;
  for (int o = rg; o < n_out; o += NRG) {
    const int u = s_src_of_out[o];
    const int64_t src_off = in_seq + (int64_t)u * in.stride_s;
    const int64_t dst_off = out_seq + (int64_t)o * out.stride_s;
    const int nmem = (u & 1) ? s_cnt[u >> 1] : 0;
    const int du = dseq ? dseq[u] : 1;
    if (nmem == 0) {  // untouched token: bit copy
      *reinterpret_cast<uint4*>(K_out + dst_off) = *reinterpret_cast<const uint4*>(K + src_off);
      *reinterpret_cast<uint4*>(V_out + dst_off) = *reinterpret_cast<const uint4*>(V + src_off);
      if (piece == 0) dout[o] = du;
      continue;
    }
    float x[E], y[E];
    Acc ak[E], av[E];
    Row<T>::load(K + src_off, x);
    Row<T>::load(V + src_off, y);
    {
      const Acc w = (Acc)du;
#pragma unroll
      for (int e = 0; e < E; ++e) { ak[e] = w * (Acc)x[e]; av[e] = w * (Acc)y[e]; }
    }
    int ndeg = du;
    const int first = s_start[u >> 1];
    for (int q = 0; q < nmem; ++q) {
      const int ua = 2 * (int)s_members[first + q];
      const int da = dseq ? dseq[ua] : 1;
      const int64_t a_off = in_seq + (int64_t)ua * in.stride_s;
      Row<T>::load(K + a_off, x);
      Row<T>::load(V + a_off, y);
      const Acc w = (Acc)da;
#pragma unroll
      for (int e = 0; e < E; ++e) { ak[e] += w * (Acc)x[e]; av[e] += w * (Acc)y[e]; }
      ndeg += da;
    }
    Row<T>::store_div(K_out + dst_off, ak, ndeg);
    Row<T>::store_div(V_out + dst_off, av, ndeg);
    if (piece == 0) dout[o] = ndeg;
  }
}

__global__ void compose_kernel(int32_t* __restrict__ assign, const int32_t* __restrict__ map, int seq0,
                               int map_len, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  const int64_t bh = e / seq0;
  assign[e] = map[bh * map_len + assign[e]];
}

__global__ void copy_rows_kernel(const unsigned char* __restrict__ src, TensorView in,
                                 unsigned char* __restrict__ dst, TensorView out, int seq, int pieces_per_row,
                                 int elem_bytes, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  const int piece = (int)(e % pieces_per_row);
  const int64_t row = e / pieces_per_row;
  const int t = (int)(row % seq), bh = (int)(row / seq);
  const int64_t so = (in.seq_base(bh) + (int64_t)t * in.stride_s) * elem_bytes + piece * 16;
  const int64_t dof = (out.seq_base(bh) + (int64_t)t * out.stride_s) * elem_bytes + piece * 16;
  *reinterpret_cast<uint4*>(dst + dof) = *reinterpret_cast<const uint4*>(src + so);
}

__global__ void fill_deg_kernel(const int32_t* __restrict__ deg_in, int32_t* __restrict__ deg_out,
                                int64_t out_stride, int32_t* __restrict__ assign, int seq, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  const int t = (int)(e % seq);
  const int64_t bh = e / seq;
  deg_out[bh * out_stride + t] = deg_in ? deg_in[e] : 1;
  if (assign) assign[e] = t;
}

template <typename T, int D>
hipError_t launch_merge_t(const void* K, const void* V, const int32_t* deg_in, TensorView in, int n_bh,
                          int seq, int chunk, float r, const int32_t* dst_local, const float* score,
                          void* K_out, void* V_out, int32_t* deg_out, TensorView out,
                          int64_t deg_out_stride, int32_t* map_out, hipStream_t st) {
  const int n_chunks = div_up(seq, chunk);
  const int64_t total = (int64_t)n_bh * n_chunks;
  if (total > (1 << 30)) return hipErrorInvalidValue;
  ScopedTimer t(sizeof(T) == 2 ? "merge_bf16" : "merge_f32", st);
  hipLaunchKernelGGL((merge_kernel<T, D>), dim3((int)total), dim3(kThreads), 0, st,
                     static_cast<const T*>(K), static_cast<const T*>(V), deg_in, in, seq, chunk, n_chunks,
                     r, dst_local, score, static_cast<T*>(K_out), static_cast<T*>(V_out), deg_out, out,
                     deg_out_stride, map_out);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_merge(const void* K, const void* V, const int32_t* deg_in, int dtype, int dim,
                        TensorView in, int n_bh, int seq, int chunk, float r,
                        const int32_t* dst_local, const float* score, void* K_out, void* V_out,
                        int32_t* deg_out, TensorView out, int64_t deg_out_stride, int out_seq,
                        int32_t* map_out, hipStream_t st) {
  (void)out_seq;
#define CKV_MERGE(T, DD)                                                                             \
  return launch_merge_t<T, DD>(K, V, deg_in, in, n_bh, seq, chunk, r, dst_local, score, K_out, V_out, \
                               deg_out, out, deg_out_stride, map_out, st)
  if (dtype == CKV_BF16) {
    if (dim == 128) CKV_MERGE(__bf16, 128);
    if (dim == 64) CKV_MERGE(__bf16, 64);
  } else {
    if (dim == 128) CKV_MERGE(float, 128);
    if (dim == 64) CKV_MERGE(float, 64);
    if (dim == 32) CKV_MERGE(float, 32);
    if (dim == 16) CKV_MERGE(float, 16);
  }
#undef CKV_MERGE
  return hipErrorInvalidValue;
}

hipError_t launch_compose(int32_t* assign, const int32_t* map, int n_bh, int seq0, int map_len,
                          hipStream_t st) {
  const int64_t total = (int64_t)n_bh * seq0;
  ScopedTimer t("compose_assign", st);
  hipLaunchKernelGGL(compose_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, assign, map,
                     seq0, map_len, total);
  return hipGetLastError();
}

hipError_t launch_copy_rows(const void* src, TensorView in, void* dst, TensorView out, int n_bh, int seq,
                            int row_bytes, int elem_bytes, hipStream_t st) {
  const int ppr = row_bytes / 16;
  const int64_t total = (int64_t)n_bh * seq * ppr;
  ScopedTimer t("copy_rows", st);
  hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                     static_cast<const unsigned char*>(src), in, static_cast<unsigned char*>(dst), out, seq,
                     ppr, elem_bytes, total);
  return hipGetLastError();
}

hipError_t launch_fill_deg(const int32_t* deg_in, int32_t* deg_out, int64_t out_stride, int32_t* assign,
                           int n_bh, int seq, hipStream_t st) {
  const int64_t total = (int64_t)n_bh * seq;
  ScopedTimer t("fill_deg", st);
  hipLaunchKernelGGL(fill_deg_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, deg_in,
                     deg_out, out_stride, assign, seq, total);
  return hipGetLastError();
}

}  // namespace ckv
