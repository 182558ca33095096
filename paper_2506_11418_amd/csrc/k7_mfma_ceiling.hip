// Measurement aid, not part of the hot path: what rate of bf16 MFMA 32x32x16 instructions this chip
// sustains when nothing else limits them, so that the similarity kernel's MFMA fraction can be read
// against what the hardware delivers under its power management and not only against the nominal
// peak (clock x units).  One workgroup per CU; every wave keeps NT independent accumulator chains
// busy for `iters` rounds of 8 k-steps, with operands that hold pseudo-random finite bf16 values (an
// all-zero operand would draw less power and flatter the result):
//   mode 0  operands stay in registers;
//   mode 1  one B fragment is read from LDS per 2 MFMAs (64 A rows per wave: the similarity kernel's ratio);
//   mode 2  one B fragment from LDS per 4 MFMAs (128 A rows per wave).
#include "ckv_internal.h"
#include "ckv_device.h"

namespace ckv {
namespace {

constexpr int kCeilLds = 32768;

template <int MODE, int NWAVES>
__global__ __launch_bounds__(NWAVES * 64, 1) void mfma_ceiling_kernel(const uint4* __restrict__ src, float* __restrict__ out,
                                                                      int iters) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  constexpr int NT = (MODE == 2) ? 4 : 2;
  for (int i = tid; i < 24576 / 16; i += NWAVES * 64) reinterpret_cast<uint4*>(smem)[i] = src[i];
  __syncthreads();
  bf16x8 a[NT][8];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int s = 0; s < 8; ++s) a[t][s] = __builtin_bit_cast(bf16x8, src[(tid * 37 + t * 8 + s) & 1023]);
  f32x16 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = f32x16{0};
  bf16x8 b[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) b[s] = __builtin_bit_cast(bf16x8, src[(tid + s * 64) & 1023]);
  int off = lane * 16;                       // 16 KiB of LDS are walked in two halves: every access stays below 24 KiB
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      if (MODE >= 1) b[s] = *reinterpret_cast<const bf16x8*>(smem + off + s * 1024);
#pragma unroll
      for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[s], a[t][s], acc[t], 0, 0, 0);
    }
    if (MODE >= 1) off ^= 8192;
  }
  float r = 0.f;
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[t][i];
  out[blockIdx.x * NWAVES * 64 + tid] = r;
}

__global__ void mfma_ceiling_fill_kernel(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  uint32_t x = 12345u + 2654435761u * (uint32_t)i;      // bf16 pairs with exponents near 1.0 and random mantissa / sign
  x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
  const uint32_t lo = 0x3f00u | ((x >> 8) & 0x80ffu), hi = 0x3f00u | ((x >> 16) & 0x80ffu);
  p[i] = lo | (hi << 16);
}

template <int MODE, int NWAVES>
hipError_t run(const uint4* src, float* out, int iters, int n_cu, hipStream_t st) {
  static KernelSetup setup;
  if (hipError_t e = kernel_setup(reinterpret_cast<const void*>(&mfma_ceiling_kernel<MODE, NWAVES>), kCeilLds, setup); e != hipSuccess)
    return e;
  hipLaunchKernelGGL((mfma_ceiling_kernel<MODE, NWAVES>), dim3(n_cu), dim3(NWAVES * 64), kCeilLds, st, src, out, iters);
  return hipGetLastError();
}

}  // namespace
}  // namespace ckv

extern "C" int ckv_bench_mfma_ceiling(int32_t mode, int32_t waves_per_cu, int32_t iters, void* scratch, size_t scratch_bytes,
                                      double* flops, void* hip_stream) {
  using namespace ckv;
  if (!scratch || !flops || iters <= 0) return CKV_EINVAL;
  if (((uintptr_t)scratch) % 256) return CKV_EALIGN;
  if (mode < 0 || mode > 2 || (waves_per_cu != 4 && waves_per_cu != 8) || (mode == 2 && waves_per_cu != 4)) return CKV_EUNSUPPORTED;
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
    (void)hipGetLastError();
    return CKV_EHIP;
  }
  const size_t src_bytes = 65536, out_bytes = (size_t)n_cu * 512 * sizeof(float);
  if (scratch_bytes < src_bytes + out_bytes) return CKV_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint32_t* src = static_cast<uint32_t*>(scratch);
  float* out = reinterpret_cast<float*>(static_cast<unsigned char*>(scratch) + src_bytes);
  hipLaunchKernelGGL(mfma_ceiling_fill_kernel, dim3(64), dim3(256), 0, st, src, 16384);
  hipError_t e = hipGetLastError();
  const uint4* s4 = reinterpret_cast<const uint4*>(src);
  ScopedTimer t("mfma_ceiling", st);
  if (e == hipSuccess) {
    if (mode == 0 && waves_per_cu == 8) e = run<0, 8>(s4, out, iters, n_cu, st);
    else if (mode == 0) e = run<0, 4>(s4, out, iters, n_cu, st);
    else if (mode == 1 && waves_per_cu == 8) e = run<1, 8>(s4, out, iters, n_cu, st);
    else if (mode == 1) e = run<1, 4>(s4, out, iters, n_cu, st);
    else e = run<2, 4>(s4, out, iters, n_cu, st);
  }
  if (e != hipSuccess) { (void)hipGetLastError(); return CKV_EHIP; }
  const int nt = mode == 2 ? 4 : 2;
  *flops = (double)n_cu * waves_per_cu * (double)iters * 8.0 * nt * 32768.0;
  return CKV_OK;
}
