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
// looked up once per device and kept in g_scratch[].  Layout: kCounterBytes of arrival counters (one
// int32 per (batch, KV head)), then the split partials.  The counters have a place of their own,
// whatever the shape of a call: they are zero when the code object is loaded, every call leaves the
// ones it used at zero again (the merging workgroup resets them), and no call's partials ever reach
// them, so nothing has to be cleared between calls of different shapes, nor by a recorded graph
// that is replayed after calls of other shapes.
constexpr size_t kCounterBytes = 64 * 1024;
static_assert(kCounterBytes % 256 == 0 && kCounterBytes < CKV_NOALLOC_SCRATCH_BYTES, "scratch layout");
static __device__ __align__(256) unsigned char scratch[CKV_NOALLOC_SCRATCH_BYTES];

std::mutex g_lock;
void* g_scratch[kMaxDevices];   // device address of `scratch` per device, NULL until its first call

}  // namespace
}  // namespace ckv

using namespace ckv;

extern "C" int ckv_decode_attn_noalloc(const void* q, int32_t q_heads, const void* K, const void* V,
                                       const ckv_layout* kv, const int32_t* lens, const int32_t* deg, float scale,
                                       void* o, int32_t o_dtype, void* hip_stream) {
  size_t need = 0;
  int st = ckv_decode_attn_workspace(kv, q_heads, &need);   // validates the layout and q_heads
  if (st != CKV_OK) return st;
  const size_t counters = attn_counter_bytes(kv->batch, kv->heads);
  if (counters > kCounterBytes || need - counters > CKV_NOALLOC_SCRATCH_BYTES - kCounterBytes) return CKV_EWORKSPACE;
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
  unsigned char* base = nullptr;
  {
    std::lock_guard<std::mutex> g(g_lock);
    if (!g_scratch[dev]) {   // first call on this device: its own copy of the array, at its own address
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return CKV_EHIP; }
      g_scratch[dev] = p;
    }
    base = static_cast<unsigned char*>(g_scratch[dev]);
  }
  hipError_t e = launch_decode_attn(q, q_heads, K, V, kv->dtype, kv->dim,
                                    TensorView{kv->stride_b, kv->stride_h, kv->stride_s, kv->heads,
                                               kv->deg_stride ? kv->deg_stride : (int64_t)kv->seq},
                                    kv->batch, kv->heads, kv->seq, lens, deg, scale, o, o_dtype, base + kCounterBytes,
                                    PagedView{nullptr, 0, 0, 0}, s, reinterpret_cast<int32_t*>(base));
  if (e == hipSuccess) return CKV_OK;
  (void)hipGetLastError();
  return (e == hipErrorInvalidValue) ? CKV_EUNSUPPORTED : CKV_EHIP;
}
