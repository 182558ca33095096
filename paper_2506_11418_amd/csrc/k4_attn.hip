// Decode attention over a (compressed) KV cache (Eq. 3; Algorithm 1, decode line):
//   o_h = softmax(q_h K^T * scale + ln N) V,   one query token, G query heads per KV head.
// Split along the sequence: every workgroup streams a contiguous slice of K and V once with
// 16-byte loads (one row per group of row_bytes/16 lanes), serves all G query heads of its KV head
// from registers, keeps an online softmax in the exp2 domain, and writes (max, sum, o) partials;
// a second small kernel merges the partials with the usual log-sum-exp rescaling.
#include "ckv_internal.h"

namespace ckv {
namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

template <typename T>
struct Elems;
template <>
struct Elems<__bf16> {
  static constexpr int E = 8;
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
  __device__ static void load(const float* p, float* x) {
    const float4 u = *reinterpret_cast<const float4*>(p);
    x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w;
  }
};

__device__ inline uint16_t f32_to_bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// partial layout: o_part[((b*Hkv + kvh)*S + split)*G + g][D], ml_part[...][2] = (max, sum)
template <typename T, int D, int G>
__global__ __launch_bounds__(kThreads) void attn_partial_kernel(
    const T* __restrict__ q, const T* __restrict__ K, const T* __restrict__ V, TensorView kv, int kv_heads,
    int seq, const int32_t* __restrict__ lens, const int32_t* __restrict__ deg, float scale_log2e,
    int n_splits, int span, float* __restrict__ o_part, float* __restrict__ ml_part) {
  constexpr int E = Elems<T>::E;
  constexpr int LPR = D / E;
  constexpr int NRG = kThreads / LPR;
  __shared__ float s_m[NRG][G];
  __shared__ float s_l[NRG][G];
  __shared__ float s_o[NRG][D];

  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, rg = tid / LPR, piece = tid % LPR;
  const int len = lens ? min(lens[b], seq) : seq;
  const int t0 = split * span, t1 = min(t0 + span, len);
  const int64_t base = (int64_t)b * kv.stride_b + (int64_t)kvh * kv.stride_h + piece * E;
  const int32_t* dseq = deg ? deg + ((int64_t)b * kv_heads + kvh) * seq : nullptr;

  float qf[G][E];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float x[E];
    Elems<T>::load(q + ((int64_t)b * kv_heads * G + kvh * G + g) * D + piece * E, x);
#pragma unroll
    for (int e = 0; e < E; ++e) qf[g][e] = x[e] * scale_log2e;
  }
  float m[G], l[G], acc[G][E];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) acc[g][e] = 0.f;
  }

  for (int t = t0 + rg; t < t1; t += NRG) {
    float kx[E], vx[E];
    Elems<T>::load(K + base + (int64_t)t * kv.stride_s, kx);
    Elems<T>::load(V + base + (int64_t)t * kv.stride_s, vx);
    const float bias = dseq ? __log2f((float)dseq[t]) : 0.f;
    float z[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < E; ++e) d = fmaf(qf[g][e], kx[e], d);
      z[g] = d;
    }
#pragma unroll
    for (int s = 1; s < LPR; s <<= 1) {
#pragma unroll
      for (int g = 0; g < G; ++g) z[g] += __shfl_xor(z[g], s);
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float zg = z[g] + bias;
      const float mn = fmaxf(m[g], zg);
      const float alpha = exp2f(m[g] - mn);
      const float p = exp2f(zg - mn);
      l[g] = l[g] * alpha + p;
#pragma unroll
      for (int e = 0; e < E; ++e) acc[g][e] = fmaf(acc[g][e], alpha, p * vx[e]);
      m[g] = mn;
    }
  }

  // ---- merge the NRG row groups of this workgroup ---------------------------------------------
  if (piece == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) { s_m[rg][g] = m[g]; s_l[rg][g] = l[g]; }
  }
  __syncthreads();
  const int64_t pbase = (((int64_t)b * kv_heads + kvh) * n_splits + split) * G;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float M = -INFINITY;
    for (int r2 = 0; r2 < NRG; ++r2) M = fmaxf(M, s_m[r2][g]);
    const float f = (m[g] == -INFINITY) ? 0.f : exp2f(m[g] - M);
#pragma unroll
    for (int e = 0; e < E; ++e) s_o[rg][piece * E + e] = acc[g][e] * f;
    __syncthreads();
    if (tid < D) {
      float sum = 0.f;
      for (int r2 = 0; r2 < NRG; ++r2) sum += s_o[r2][tid];
      o_part[(pbase + g) * D + tid] = sum;
    }
    if (tid == 0) {
      float L = 0.f;
      for (int r2 = 0; r2 < NRG; ++r2) {
        const float mr = s_m[r2][g];
        L += (mr == -INFINITY) ? 0.f : s_l[r2][g] * exp2f(mr - M);
      }
      ml_part[(pbase + g) * 2] = M;
      ml_part[(pbase + g) * 2 + 1] = L;
    }
    __syncthreads();
  }
}

template <int G>
__global__ void attn_combine_kernel(const float* __restrict__ o_part, const float* __restrict__ ml_part,
                                    int kv_heads, int n_splits, int dim, void* __restrict__ o, int o_dtype) {
  const int hq = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
  const int kvh = hq / G, g = hq % G;
  const int64_t pbase = ((int64_t)b * kv_heads + kvh) * n_splits;
  float M = -INFINITY;
  for (int s = 0; s < n_splits; ++s) M = fmaxf(M, ml_part[((pbase + s) * G + g) * 2]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const int64_t idx = (pbase + s) * G + g;
    const float ms = ml_part[idx * 2];
    if (ms == -INFINITY) continue;
    const float f = exp2f(ms - M);
    den += ml_part[idx * 2 + 1] * f;
    if (d < dim) num += o_part[idx * dim + d] * f;
  }
  if (d >= dim) return;
  const float res = den > 0.f ? num / den : 0.f;
  const int64_t oi = ((int64_t)b * kv_heads * G + hq) * dim + d;
  if (o_dtype == CKV_BF16) reinterpret_cast<uint16_t*>(o)[oi] = f32_to_bf16_rne(res);
  else reinterpret_cast<float*>(o)[oi] = res;
}

template <typename T, int D, int G>
hipError_t launch_attn_t(const void* q, const void* K, const void* V, TensorView kv, int n_b, int kv_heads,
                         int seq, const int32_t* lens, const int32_t* deg, float scale, void* o, int o_dtype,
                         void* workspace, hipStream_t st) {
  const int n_splits = attn_splits(n_b, kv_heads, seq);
  const int span = div_up(seq, n_splits);
  float* o_part = static_cast<float*>(workspace);
  float* ml_part = o_part + (size_t)n_b * kv_heads * n_splits * G * D;
  {
    ScopedTimer t(sizeof(T) == 2 ? "attn_partial_bf16" : "attn_partial_f32", st);
    hipLaunchKernelGGL((attn_partial_kernel<T, D, G>), dim3(n_splits, kv_heads, n_b), dim3(kThreads), 0, st,
                       static_cast<const T*>(q), static_cast<const T*>(K), static_cast<const T*>(V), kv,
                       kv_heads, seq, lens, deg, scale * kLog2e, n_splits, span, o_part, ml_part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  ScopedTimer t("attn_combine", st);
  hipLaunchKernelGGL((attn_combine_kernel<G>), dim3(kv_heads * G, n_b), dim3(D < 64 ? 64 : D), 0, st, o_part,
                     ml_part, kv_heads, n_splits, D, o, o_dtype);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_attn_g(int G, const void* q, const void* K, const void* V, TensorView kv, int n_b,
                         int kv_heads, int seq, const int32_t* lens, const int32_t* deg, float scale, void* o,
                         int o_dtype, void* workspace, hipStream_t st) {
  switch (G) {
    case 1: return launch_attn_t<T, D, 1>(q, K, V, kv, n_b, kv_heads, seq, lens, deg, scale, o, o_dtype, workspace, st);
    case 2: return launch_attn_t<T, D, 2>(q, K, V, kv, n_b, kv_heads, seq, lens, deg, scale, o, o_dtype, workspace, st);
    case 4: return launch_attn_t<T, D, 4>(q, K, V, kv, n_b, kv_heads, seq, lens, deg, scale, o, o_dtype, workspace, st);
    case 8: return launch_attn_t<T, D, 8>(q, K, V, kv, n_b, kv_heads, seq, lens, deg, scale, o, o_dtype, workspace, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace

int attn_splits(int n_b, int kv_heads, int seq) {
  // enough workgroups to fill 256 CUs several times over, but at least 256 tokens per slice
  const int64_t bh = (int64_t)n_b * kv_heads;
  int want = (int)((2048 + bh - 1) / bh);
  const int cap = (seq + 255) / 256;
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  return want;
}

size_t attn_workspace_bytes(int n_b, int kv_heads, int q_heads, int dim, int seq) {
  const size_t rows = (size_t)n_b * q_heads * attn_splits(n_b, kv_heads, seq);
  return rows * (dim + 2) * sizeof(float);
}

hipError_t launch_decode_attn(const void* q, int q_heads, const void* K, const void* V, int dtype, int dim,
                              TensorView kv, int n_b, int kv_heads, int seq, const int32_t* lens,
                              const int32_t* deg, float scale, void* o, int o_dtype, void* workspace,
                              hipStream_t st) {
  const int G = q_heads / kv_heads;
#define CKV_ATTN(T, DD) \
  return launch_attn_g<T, DD>(G, q, K, V, kv, n_b, kv_heads, seq, lens, deg, scale, o, o_dtype, workspace, st)
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
