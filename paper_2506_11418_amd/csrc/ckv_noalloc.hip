// ckv_decode_attn for callers that may not allocate device memory (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc): the split partials and arrival counters
// live in a device array that is part of the library's code object instead of a caller-supplied
// workspace.  Every GPU the library runs on holds its own copy of the array until the process ends.
#include <math.h>

#include <mutex>

#include "ckv_internal.h"

namespace ckv {
namespace {

// In host code this name is only a handle for hipGetSymbolAddress: the array's device address is
// looked up once per device and kept in g_scratch[].
static __device__ __align__(256) unsigned char scratch[CKV_NOALLOC_SCRATCH_BYTES];

struct DeviceScratch {
  void* ptr = nullptr;          // device address of `scratch` on this device
  size_t counters_zero = 0;     // leading bytes known to hold zeroed arrival counters
};
std::mutex g_lock;
DeviceScratch g_scratch[kMaxDevices];

__global__ void zero_words_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

}  // namespace
}  // namespace ckv

using namespace ckv;

extern "C" int ckv_decode_attn_noalloc(const void* q, int32_t q_heads, const void* K, const void* V,
                                       const ckv_layout* kv, const int32_t* lens, const int32_t* deg, float scale,
                                       void* o, int32_t o_dtype, void* hip_stream) {
  size_t need = 0;
  int st = ckv_decode_attn_workspace(kv, q_heads, &need);   // validates the layout and q_heads
  if (st != CKV_OK) return st;
  if (need > CKV_NOALLOC_SCRATCH_BYTES) return CKV_EWORKSPACE;
  if (!q || !K || !V || !o) return CKV_EINVAL;
  if (o_dtype != CKV_F32 && o_dtype != CKV_BF16) return CKV_EINVAL;
  if (((uintptr_t)q) % 16 || ((uintptr_t)K) % 16 || ((uintptr_t)V) % 16 || ((uintptr_t)o) % 4 ||
      ((uintptr_t)lens) % 4 || ((uintptr_t)deg) % 4)
    return CKV_EALIGN;
  const int G = q_heads / kv->heads;
  if (G != 1 && G != 2 && G != 4 && G != 8) return CKV_EUNSUPPORTED;
  if (kv->dtype == CKV_BF16 ? !(kv->dim == 64 || kv->dim == 128) : !(kv->dim == 32 || kv->dim == 64 || kv->dim == 128))
    return CKV_EUNSUPPORTED;
  if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)kv->dim);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return CKV_EHIP; }
  if (dev < 0 || dev >= kMaxDevices) return CKV_EUNSUPPORTED;
  void* ws = nullptr;
  {
    std::lock_guard<std::mutex> g(g_lock);
    DeviceScratch& d = g_scratch[dev];
    if (!d.ptr) {   // first call on this device: its own copy of the array, at its own address
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return CKV_EHIP; }
      d.ptr = p;
      d.counters_zero = 0;
    }
    ws = d.ptr;
    // The arrival counters sit at the start of the scratch and are zero again after every call; a
    // call with more (batch, KV head) pairs than the one before reaches into what that one used
    // for partial results, so its counters are cleared first (a fill kernel on the caller's stream,
    // not a memset: the call may be under graph capture).
    const size_t cb = attn_counter_bytes(kv->batch, kv->heads);
    if (cb > d.counters_zero) {
      const int n = (int)(cb / sizeof(int32_t));
      hipLaunchKernelGGL(zero_words_kernel, dim3((n + 255) / 256), dim3(256), 0, s, static_cast<int32_t*>(ws), n);
      if (hipGetLastError() != hipSuccess) return CKV_EHIP;
    }
    d.counters_zero = cb;
  }
  hipError_t e = launch_decode_attn(q, q_heads, K, V, kv->dtype, kv->dim,
                                    TensorView{kv->stride_b, kv->stride_h, kv->stride_s, kv->heads,
                                               kv->deg_stride ? kv->deg_stride : (int64_t)kv->seq},
                                    kv->batch, kv->heads, kv->seq, lens, deg, scale, o, o_dtype, ws,
                                    PagedView{nullptr, 0, 0, 0}, s);
  if (e == hipSuccess) return CKV_OK;
  (void)hipGetLastError();
  return (e == hipErrorInvalidValue) ? CKV_EUNSUPPORTED : CKV_EHIP;
}
