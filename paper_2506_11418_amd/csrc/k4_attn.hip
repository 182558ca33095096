// Decode attention over a (compressed) KV cache (Eq. 3; Algorithm 1, decode line):
//   o_h = softmax(q_h K^T * scale + ln N) V,   one query token, G query heads per KV head.
// Split along the sequence: every workgroup streams a contiguous slice of K and V once with
// 16-byte loads (one row per group of row_bytes/16 lanes), serves all G query heads of its KV head
// from registers, keeps an online softmax in the exp2 domain, and writes (max, sum, o) partials.
// The slice that finishes last for a (batch, KV head) - found with one counter word per pair in
// the workspace, which that workgroup puts back to zero - merges the partials of all slices with
// the usual log-sum-exp rescaling, in slice order, so the result does not depend on which one that
// is.  One launch per call; nothing in it is a memset.
#include <type_traits>

#include "ckv_internal.h"
#include "ckv_device.h"

namespace ckv {
namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

template <typename T>
struct Elems;
template <>
struct Elems<__bf16> {
  static constexpr int E = 8;
  typedef uint4 Raw;
  __device__ static Raw load_raw(const __bf16* p) { return ldg16_stream(p); }
  __device__ static void unpack(const Raw& u, float* x) {
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(w[i] << 16);
      x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  // q.k over this lane's 8 elements: packed bf16 pairs straight into v_dot2 (products exact,
  // fp32 accumulation), no unpacking of the key
  typedef uint4 Q;
  __device__ static Q load_q(const __bf16* p) { return *reinterpret_cast<const uint4*>(p); }
  __device__ static float dot(const Q& qv, const Raw& kv) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    const uint32_t a[4] = {qv.x, qv.y, qv.z, qv.w}, b[4] = {kv.x, kv.y, kv.z, kv.w};
    float d = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a[i]), __builtin_bit_cast(bf16x2, b[i]), d, false);
    return d;
  }
  __device__ static void load(const __bf16* p, float* x) {
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(w[i] << 16);
      x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};
template <>
struct Elems<float> {
  static constexpr int E = 4;
  typedef float4 Raw;
  __device__ static Raw load_raw(const float* p) { return *reinterpret_cast<const float4*>(p); }
  __device__ static void unpack(const Raw& u, float* x) { x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w; }
  typedef float4 Q;
  __device__ static Q load_q(const float* p) { return *reinterpret_cast<const float4*>(p); }
  __device__ static float dot(const Q& a, const Raw& b) {
    return fmaf(a.w, b.w, fmaf(a.z, b.z, fmaf(a.y, b.y, a.x * b.x)));
  }
  __device__ static void load(const float* p, float* x) {
    const float4 u = *reinterpret_cast<const float4*>(p);
    x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w;
  }
};

// Sum over the LANES consecutive lanes (aligned) that share a cache row; every lane gets the sum.
// Quad steps and the mirrored half-row / row are DPP adds; 32 lanes add one cross-row exchange.
template <int LANES>
__device__ __forceinline__ float row_sum(float x) {
  auto dpp = [](float v, auto ctrl) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value,
                                                                 0xF, 0xF, true));
  };
  x += dpp(x, std::integral_constant<int, 0xB1>{});                    // lane ^ 1
  x += dpp(x, std::integral_constant<int, 0x4E>{});                    // lane ^ 2
  if (LANES >= 8) x += dpp(x, std::integral_constant<int, 0x141>{});   // mirrored within 8
  if (LANES >= 16) x += dpp(x, std::integral_constant<int, 0x140>{});  // mirrored within 16
  if (LANES >= 32) x += __shfl_xor(x, 16);
  return x;
}

__device__ inline uint16_t f32_to_bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// Partial results travel between workgroups that may sit on different XCDs (each with its own L2)
// inside one launch.  They are written and read with device-scope relaxed atomic accesses, which go
// through to the level all XCDs share, instead of plain accesses bracketed by device-scope fences:
// such a fence writes back / invalidates a whole L2, and one per workgroup cost this kernel a
// factor of three.
__device__ __forceinline__ void store_shared_f32(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_shared_f32(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 2^x for x <= 0 as the bare hardware instruction (1 ulp; results below 2^-126 come out as zero).
// The library routine wraps it in a range fix-up for denormal results, five more instructions per
// call, which in the streaming loop is a fifth of all vector work and buys nothing for a softmax weight.
__device__ __forceinline__ float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }

// partial layout: o_part[((b*Hkv + kvh)*S + split)*G + g][D], ml_part[...][2] = (max, sum)
//
// Thread mapping: LPR = row_bytes/16 lanes share one cache row ("row group"); a wave holds 64/LPR
// row groups, so one wave-wide 16-byte load covers 64/LPR consecutive rows = 1 KiB contiguous.
// Every row group takes kUnroll tokens per iteration: their K and V loads are all issued before
// the first use (bytes in flight hide HBM latency), the logits of the kUnroll tokens share one
// running-max update, so the accumulators are rescaled once per kUnroll tokens.
constexpr int kUnroll = 4;
constexpr int kMaxSplits = 1024;    // slices per sequence: the merge keeps one weight per slice and head in LDS
constexpr int kMaxTableLds = 2048;   // block-table entries of one slice kept in LDS (paged caches)

// PAGED: K, V are a block pool [n_blocks, heads, block_size, dim] (kv.stride_s = dim, kv.stride_h =
// block_size*dim: the tokens of one head are contiguous inside a block), token t of sequence b
// lives in block table[b][t / block_size] at offset t % block_size, degrees in a pool
// [n_blocks, heads, block_size].  A table entry outside the pool masks its tokens.
template <typename T, int D, int G, bool PAGED>
__global__ __launch_bounds__(kThreads, G <= 4 ? 3 : 2) void attn_partial_kernel(
    const T* __restrict__ q, const T* __restrict__ K, const T* __restrict__ V, TensorView kv, int kv_heads,
    int seq, const int32_t* __restrict__ lens, const int32_t* __restrict__ deg, float scale_log2e,
    int n_splits, int span, float* __restrict__ o_part, float* __restrict__ ml_part,
    int32_t* __restrict__ arrived, void* __restrict__ o, int o_dtype, PagedView paged) {
  constexpr int E = Elems<T>::E;
  constexpr int LPR = D / E;
  constexpr int NRG = kThreads / LPR;
  constexpr int U = kUnroll;
  __shared__ float s_m[NRG][G];
  __shared__ float s_l[NRG][G];
  constexpr int GG = (G < 4) ? G : 4;   // query heads merged per pass of the final reduction
  // staging rows of the workgroup's reduction; later the slice weights [G][kMaxSplits] of the merge
  constexpr int kStageFloats = GG * NRG * D, kWeightFloats = G * kMaxSplits;
  __shared__ float s_raw[kStageFloats > kWeightFloats ? kStageFloats : kWeightFloats];
  float (*s_o)[NRG][D] = reinterpret_cast<float (*)[NRG][D]>(s_raw);

  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, rg = tid / LPR, piece = tid % LPR;
  const int len = lens ? min(lens[b], seq) : seq;
  const int t0 = split * span, t1 = min(t0 + span, len);
  const int64_t base = PAGED ? piece * E : (int64_t)b * kv.stride_b + (int64_t)kvh * kv.stride_h + piece * E;
  const T* Kp = K + base;
  const T* Vp = V + base;
  const int32_t* dseq = !deg ? nullptr : PAGED ? deg : deg + ((int64_t)b * kv_heads + kvh) * kv.deg_stride;
  const int32_t* tbl = PAGED ? paged.table + (int64_t)b * paged.max_blocks : nullptr;
  const int bs_mask = (1 << paged.shift) - 1;
  // the slice's blocks go to LDS first, each as the pool row ((block, head) pair times block size)
  // its first token of this head sits in, or -1 for an entry outside the pool: a row's address then
  // needs no second trip to memory and one add (the host sizes the slices so that their table
  // entries fit, and refuses pools of 2^31 rows or more)
  __shared__ int32_t s_tbl[PAGED ? kMaxTableLds : 1];
  const int blk0 = t0 >> paged.shift;
  if (PAGED && t0 < t1) {
    const int n_ent = min(((t1 - 1) >> paged.shift) - blk0 + 1, kMaxTableLds);
    for (int i = tid; i < n_ent; i += kThreads) {
      const int blk = tbl[blk0 + i];
      s_tbl[i] = ((unsigned)blk < (unsigned)paged.n_blocks) ? ((blk * kv_heads + kvh) << paged.shift) : -1;
    }
    __syncthreads();
  }

  typename Elems<T>::Q qv[G];
#pragma unroll
  for (int g = 0; g < G; ++g)
    qv[g] = Elems<T>::load_q(q + ((int64_t)b * kv_heads * G + kvh * G + g) * D + piece * E);
  float m[G], l[G], acc[G][E];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) acc[g][e] = 0.f;
  }

  // token of (iteration, slot u) for this row group: tb + u*NRG + rg.  The loads of iteration
  // i+1 are issued before iteration i is consumed (two register sets, software pipeline).
  struct Stage {
    typename Elems<T>::Raw kr[U], vr[U];
    int dg[U];
  };
  auto issue = [&](Stage& st, int tb) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tc = min(tb + u * NRG + rg, t1 - 1);   // clamp: always a valid row, masked at use
      if (PAGED) {
        const int row0 = s_tbl[min((tc >> paged.shift) - blk0, kMaxTableLds - 1)];
        const bool in_pool = row0 >= 0;
        // row 0 when outside the pool: always a valid address, masked through the degree
        const int row = in_pool ? row0 + (tc & bs_mask) : 0;
        st.kr[u] = Elems<T>::load_raw(Kp + (int64_t)row * kv.stride_s);
        st.vr[u] = Elems<T>::load_raw(Vp + (int64_t)row * kv.stride_s);
        const int d = dseq ? dseq[row] : 1;
        st.dg[u] = in_pool ? d : 0;
      } else {
        st.kr[u] = Elems<T>::load_raw(Kp + (int64_t)tc * kv.stride_s);
        st.vr[u] = Elems<T>::load_raw(Vp + (int64_t)tc * kv.stride_s);
        st.dg[u] = dseq ? dseq[tc] : 1;
      }
    }
  };
  auto consume = [&](const Stage& st, int tb) {
    float z[U][G];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int g = 0; g < G; ++g) z[u][g] = row_sum<LPR>(Elems<T>::dot(qv[g], st.kr[u]));
      const float lb = dseq ? __log2f((float)st.dg[u]) : 0.f;
      const bool ok = (tb + u * NRG + rg) < t1 && (!PAGED || st.dg[u] > 0);
#pragma unroll
      for (int g = 0; g < G; ++g) z[u][g] = ok ? fmaf(z[u][g], scale_log2e, lb) : -INFINITY;
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mn = m[g];
#pragma unroll
      for (int u = 0; u < U; ++u) mn = fmaxf(mn, z[u][g]);
      // a row group that has seen no valid token yet keeps mn = -inf: subtract 0 instead, so that
      // exp2(-inf) = 0 comes out rather than NaN
      const float ref = (mn == -INFINITY) ? 0.f : mn;
      const float alpha = exp2_raw(m[g] - ref);
      m[g] = mn;
      l[g] *= alpha;
#pragma unroll
      for (int e = 0; e < E; ++e) acc[g][e] *= alpha;
#pragma unroll
      for (int u = 0; u < U; ++u) z[u][g] = exp2_raw(z[u][g] - ref);   // now the weight p
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float vx[E];
      Elems<T>::unpack(st.vr[u], vx);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        l[g] += z[u][g];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[g][e] = fmaf(z[u][g], vx[e], acc[g][e]);
      }
    }
  };
  constexpr int STEP = NRG * U;
  if (t0 < t1) {
    Stage sa, sb;
    issue(sa, t0);
    for (int tb = t0; tb < t1; tb += 2 * STEP) {
      if (tb + STEP < t1) issue(sb, tb + STEP);
      consume(sa, tb);
      if (tb + STEP < t1) {
        if (tb + 2 * STEP < t1) issue(sa, tb + 2 * STEP);
        consume(sb, tb + STEP);
      }
    }
  }

  // ---- merge the NRG row groups of this workgroup ---------------------------------------------
  if (piece == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) { s_m[rg][g] = m[g]; s_l[rg][g] = l[g]; }
  }
  __syncthreads();
  const int64_t pbase = (((int64_t)b * kv_heads + kvh) * n_splits + split) * G;
  // GG heads at a time: every row group rescales its accumulators to the workgroup's maximum and
  // parks them in LDS, then each thread sums a few (head, channel) columns over the row groups
#pragma unroll
  for (int g0 = 0; g0 < G; g0 += GG) {
    if (g0 > 0) __syncthreads();
#pragma unroll
    for (int gg = 0; gg < GG; ++gg) {
      const int g = g0 + gg;
      float M = -INFINITY;
      for (int r2 = 0; r2 < NRG; ++r2) M = fmaxf(M, s_m[r2][g]);
      const float f = (m[g] == -INFINITY) ? 0.f : exp2f(m[g] - M);
#pragma unroll
      for (int e = 0; e < E; ++e) s_o[gg][rg][piece * E + e] = acc[g][e] * f;
    }
    __syncthreads();
    for (int idx = tid; idx < GG * D; idx += kThreads) {
      const int gg = idx / D, d = idx % D;
      float sum = 0.f;
      for (int r2 = 0; r2 < NRG; ++r2) sum += s_o[gg][r2][d];
      store_shared_f32(&o_part[(pbase + g0 + gg) * D + d], sum);
    }
    if (tid < GG) {
      const int g = g0 + tid;
      float M = -INFINITY, L = 0.f;
      for (int r2 = 0; r2 < NRG; ++r2) M = fmaxf(M, s_m[r2][g]);
      for (int r2 = 0; r2 < NRG; ++r2) {
        const float mr = s_m[r2][g];
        L += (mr == -INFINITY) ? 0.f : s_l[r2][g] * exp2f(mr - M);
      }
      store_shared_f32(&ml_part[(pbase + g) * 2], M);
      store_shared_f32(&ml_part[(pbase + g) * 2 + 1], L);
    }
  }

  // ---- the last slice of this (batch, KV head) to arrive merges them all ----------------------
  // Every thread waits until its own partial stores have been acknowledged, the workgroup meets,
  // and one thread counts the workgroup in; the workgroup that finds all others counted takes the
  // merge.  The counter is only ever touched with device-scope atomics.
  __shared__ int s_is_last;
  __builtin_amdgcn_s_waitcnt(0);          // vmcnt = lgkmcnt = expcnt = 0: the stores above are complete
  __syncthreads();
  int32_t* my_count = arrived + (b * kv_heads + kvh);
  if (tid == 0) s_is_last = (atomicAdd(my_count, 1) == n_splits - 1);
  __syncthreads();
  if (!s_is_last) return;
  // weights of the slices, per query head: a wave takes a head (two for G = 8)
  float* s_w = s_raw;                     // [G][kMaxSplits] (the staging rows are no longer needed)
  float* s_den = &s_l[0][0];              // [G]
  const int lane = tid & 63, wave = tid >> 6;
  const int64_t sbase = ((int64_t)b * kv_heads + kvh) * n_splits;
  for (int g = wave; g < G; g += kThreads / 64) {
    float mloc = -INFINITY;
    for (int sp = lane; sp < n_splits; sp += 64) mloc = fmaxf(mloc, load_shared_f32(&ml_part[((sbase + sp) * G + g) * 2]));
#pragma unroll
    for (int sh = 32; sh > 0; sh >>= 1) mloc = fmaxf(mloc, __shfl_xor(mloc, sh));
    float dloc = 0.f;
    for (int sp = lane; sp < n_splits; sp += 64) {
      const float ms = load_shared_f32(&ml_part[((sbase + sp) * G + g) * 2]);       // max of slice sp
      const float ls = load_shared_f32(&ml_part[((sbase + sp) * G + g) * 2 + 1]);   // its sum of exponentials
      const float f = (ms == -INFINITY) ? 0.f : exp2f(ms - mloc);
      s_w[g * kMaxSplits + sp] = f;
      dloc += f * ls;
    }
#pragma unroll
    for (int sh = 32; sh > 0; sh >>= 1) dloc += __shfl_xor(dloc, sh);
    if (lane == 0) s_den[g] = dloc;
  }
  __syncthreads();
  // Every thread owns NC (head, channel) columns, consecutive threads consecutive channels (a wave's
  // load is 256 contiguous bytes), and sums them over the slices in slice order: blocks of 32
  // slices with all NC * 32 loads in flight, then blocks of 8, then single slices.  Which
  // workgroup runs this never changes the order, so the bits are the same from run to run.
  constexpr int NC = (G * D + kThreads - 1) / kThreads;
  float num[NC];
  const float* col[NC];
  const float* wcol[NC];
#pragma unroll
  for (int k = 0; k < NC; ++k) {
    const int c = min(tid + k * kThreads, G * D - 1);        // clamped: threads past the last column repeat it
    num[k] = 0.f;
    col[k] = o_part + (sbase * G + c / D) * D + c % D;
    wcol[k] = s_w + (c / D) * kMaxSplits;
  }
  const int64_t pitch = (int64_t)G * D;
  auto block = [&](int s0, auto n_c) {
    constexpr int N = decltype(n_c)::value;
    float x[NC][N];
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
      for (int k = 0; k < NC; ++k) x[k][i] = load_shared_f32(col[k] + (int64_t)(s0 + i) * pitch);
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
      for (int k = 0; k < NC; ++k) num[k] = fmaf(x[k][i], wcol[k][s0 + i], num[k]);
  };
  int s0 = 0;
  for (; s0 + 32 <= n_splits; s0 += 32) block(s0, std::integral_constant<int, 32>{});
  for (; s0 + 8 <= n_splits; s0 += 8) block(s0, std::integral_constant<int, 8>{});
  for (; s0 < n_splits; ++s0) block(s0, std::integral_constant<int, 1>{});
#pragma unroll
  for (int k = 0; k < NC; ++k) {
    const int c = tid + k * kThreads;
    if (c < G * D) {
      const float den = s_den[c / D];
      const float res = den > 0.f ? num[k] / den : 0.f;
      const int64_t oi = ((int64_t)b * kv_heads + kvh) * G * D + c;
      if (o_dtype == CKV_BF16) reinterpret_cast<uint16_t*>(o)[oi] = f32_to_bf16_rne(res);
      else reinterpret_cast<float*>(o)[oi] = res;
    }
  }
  if (tid == 0) atomicExch(my_count, 0);  // the workspace is ready for the next call
}

template <typename T, int D, int G>
hipError_t launch_attn_t(const void* q, const void* K, const void* V, TensorView kv, int n_b, int kv_heads,
                         int seq, const int32_t* lens, const int32_t* deg, float scale, void* o, int o_dtype,
                         void* workspace, int32_t* counters, PagedView paged, hipStream_t st) {
  const int n_splits = attn_splits(n_b, kv_heads, seq, paged.table ? (kMaxTableLds << paged.shift) : 0);
  const int span = div_up(seq, n_splits);
  if (paged.table && span > (kMaxTableLds << paged.shift)) return hipErrorInvalidValue;
  // workspace: arrival counters (one per (batch, KV head), zero between calls) | partial outputs | (max, sum) pairs;
  // with counters kept elsewhere the partial outputs start the workspace
  int32_t* arrived = counters ? counters : static_cast<int32_t*>(workspace);
  float* o_part = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) +
                                           (counters ? 0 : attn_counter_bytes(n_b, kv_heads)));
  float* ml_part = o_part + (size_t)n_b * kv_heads * n_splits * G * D;
  ScopedTimer t(paged.table ? (sizeof(T) == 2 ? "attn_paged_bf16" : "attn_paged_f32")
                            : (sizeof(T) == 2 ? "attn_bf16" : "attn_f32"), st);
  if (paged.table)
    hipLaunchKernelGGL((attn_partial_kernel<T, D, G, true>), dim3(n_splits, kv_heads, n_b), dim3(kThreads), 0,
                       st, static_cast<const T*>(q), static_cast<const T*>(K), static_cast<const T*>(V), kv,
                       kv_heads, seq, lens, deg, scale * kLog2e, n_splits, span, o_part, ml_part, arrived, o, o_dtype,
                       paged);
  else
    hipLaunchKernelGGL((attn_partial_kernel<T, D, G, false>), dim3(n_splits, kv_heads, n_b), dim3(kThreads), 0,
                       st, static_cast<const T*>(q), static_cast<const T*>(K), static_cast<const T*>(V), kv,
                       kv_heads, seq, lens, deg, scale * kLog2e, n_splits, span, o_part, ml_part, arrived, o, o_dtype,
                       paged);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_attn_g(int G, const void* q, const void* K, const void* V, TensorView kv, int n_b,
                         int kv_heads, int seq, const int32_t* lens, const int32_t* deg, float scale, void* o,
                         int o_dtype, void* workspace, int32_t* counters, PagedView paged, hipStream_t st) {
  switch (G) {
    case 1: return launch_attn_t<T, D, 1>(q, K, V, kv, n_b, kv_heads, seq, lens, deg, scale, o, o_dtype, workspace, counters, paged, st);
    case 2: return launch_attn_t<T, D, 2>(q, K, V, kv, n_b, kv_heads, seq, lens, deg, scale, o, o_dtype, workspace, counters, paged, st);
    case 4: return launch_attn_t<T, D, 4>(q, K, V, kv, n_b, kv_heads, seq, lens, deg, scale, o, o_dtype, workspace, counters, paged, st);
    case 8: return launch_attn_t<T, D, 8>(q, K, V, kv, n_b, kv_heads, seq, lens, deg, scale, o, o_dtype, workspace, counters, paged, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace

int attn_splits(int n_b, int kv_heads, int seq, int span_limit) {
  // about two workgroups per CU (each has a fixed merge/write cost), at least 256 tokens per slice
  const int64_t bh = (int64_t)n_b * kv_heads;
  int want = (int)((512 + bh - 1) / bh);
  int cap = (seq + 255) / 256;
  if (cap > kMaxSplits) cap = kMaxSplits;   // the merge keeps one weight per slice in LDS
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  // paged caches: a slice's block-table entries must fit the kernel's LDS table
  if (span_limit > 0 && (seq + want - 1) / want > span_limit) want = (seq + span_limit - 1) / span_limit;
  if (want > kMaxSplits) want = kMaxSplits;
  return want;
}

size_t attn_counter_bytes(int n_b, int kv_heads) { return ((size_t)n_b * kv_heads * sizeof(int32_t) + 255) / 256 * 256; }

int attn_paged_span_limit(int block_size) { return kMaxTableLds * block_size; }

size_t attn_workspace_bytes(int n_b, int kv_heads, int q_heads, int dim, int seq, int span_limit) {
  // one arrival counter per (batch, KV head), then partial outputs and (max, sum) pairs per
  // (batch, query head, slice)
  const size_t rows = (size_t)n_b * q_heads * attn_splits(n_b, kv_heads, seq, span_limit);
  return attn_counter_bytes(n_b, kv_heads) + rows * (dim + 2) * sizeof(float);
}

hipError_t launch_decode_attn(const void* q, int q_heads, const void* K, const void* V, int dtype, int dim,
                              TensorView kv, int n_b, int kv_heads, int seq, const int32_t* lens,
                              const int32_t* deg, float scale, void* o, int o_dtype, void* workspace,
                              PagedView paged, hipStream_t st, int32_t* counters) {
  const int G = q_heads / kv_heads;
#define CKV_ATTN(T, DD) \
  return launch_attn_g<T, DD>(G, q, K, V, kv, n_b, kv_heads, seq, lens, deg, scale, o, o_dtype, workspace, counters, paged, st)
  if (dtype == CKV_BF16) {
    if (dim == 128) CKV_ATTN(__bf16, 128);
    if (dim == 64) CKV_ATTN(__bf16, 64);
  } else {
    if (dim == 128) CKV_ATTN(float, 128);
    if (dim == 64) CKV_ATTN(float, 64);
    if (dim == 32) CKV_ATTN(float, 32);
  }
#undef CKV_ATTN
  return hipErrorInvalidValue;
}

}  // namespace ckv
