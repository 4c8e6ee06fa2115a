// Measured ceilings of the chip, for holding the layer's kernels against something other than the
// data-sheet figures: a register-only bf16 MFMA loop (no memory traffic at all) and a plain 16 B per
// lane copy.  Measurement hooks of the C ABI; they time themselves with HIP events and block the
// host until done.
#include "../../include/gx.h"
#include "gx_kernels.h"

namespace {

using namespace gx;

// every wavefront keeps NACC independent 32x32 accumulators and issues nothing but MFMAs
constexpr int NACC = 4;
__global__ void __launch_bounds__(256) mfma_loop_kernel(float* out, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; i++) {
    a[i] = (bf16)(float)(threadIdx.x % 3);
    b[i] = (bf16)(float)(threadIdx.x % 5);
  }
  f32x16 acc[NACC];
#pragma unroll
  for (int n = 0; n < NACC; n++)
#pragma unroll
    for (int i = 0; i < 16; i++) acc[n][i] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int n = 0; n < NACC; n++) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < NACC; n++)
#pragma unroll
    for (int i = 0; i < 16; i++) s += acc[n][i];
  if (s == 12345.678f) out[0] = s;      // never true: keeps the loop alive
}

__global__ void __launch_bounds__(256) copy_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst, size_t n) {
  size_t i = blockIdx.x * (size_t)256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) dst[i] = src[i];
}

struct Events {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  bool ok = false;
  Events() { ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess; }
  ~Events() {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
  }
};

}  // namespace

extern "C" gx_status gx_peak_mfma(void* scratch, int launches, double* tflops, void* hip_stream) {
  if (!scratch || !tflops) return GX_ERR_NULL;
  if (launches < 1 || launches > 1000) return GX_ERR_SHAPE;
  if (!device_is_gfx950()) return GX_ERR_ARCH;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  Events ev;
  if (!ev.ok) return GX_ERR_LAUNCH;
  const int wgs = 1024, iters = 20000;
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(wgs), dim3(256), 0, st, static_cast<float*>(scratch), iters);   // warm-up
  if (hipEventRecord(ev.e0, st) != hipSuccess) return GX_ERR_LAUNCH;
  for (int i = 0; i < launches; i++)
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(wgs), dim3(256), 0, st, static_cast<float*>(scratch), iters);
  if (hipGetLastError() != hipSuccess || hipEventRecord(ev.e1, st) != hipSuccess ||
      hipEventSynchronize(ev.e1) != hipSuccess)
    return GX_ERR_LAUNCH;
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, ev.e0, ev.e1) != hipSuccess) return GX_ERR_LAUNCH;
  const double flop = (double)launches * wgs * 4 /* wavefronts */ * iters * NACC * 2.0 * 32 * 32 * 16;
  *tflops = flop / ((double)ms * 1e-3) / 1e12;
  return GX_OK;
}

extern "C" gx_status gx_peak_copy(const void* src, void* dst, size_t bytes, int launches, double* gbytes_per_s,
                                  void* hip_stream) {
  if (!src || !dst || !gbytes_per_s) return GX_ERR_NULL;
  if (launches < 1 || launches > 1000 || bytes < 16 || (bytes & 15)) return GX_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) return GX_ERR_ALIGN;
  if (!device_is_gfx950()) return GX_ERR_ARCH;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  Events ev;
  if (!ev.ok) return GX_ERR_LAUNCH;
  const size_t n = bytes / 16;
  const int wgs = n / 256 < 1024 ? (int)(n / 256 ? n / 256 : 1) : 1024;
  hipLaunchKernelGGL(copy_kernel, dim3(wgs), dim3(256), 0, st, static_cast<const f32x4*>(src), static_cast<f32x4*>(dst), n);
  if (hipEventRecord(ev.e0, st) != hipSuccess) return GX_ERR_LAUNCH;
  for (int i = 0; i < launches; i++)
    hipLaunchKernelGGL(copy_kernel, dim3(wgs), dim3(256), 0, st, static_cast<const f32x4*>(src), static_cast<f32x4*>(dst), n);
  if (hipGetLastError() != hipSuccess || hipEventRecord(ev.e1, st) != hipSuccess ||
      hipEventSynchronize(ev.e1) != hipSuccess)
    return GX_ERR_LAUNCH;
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, ev.e0, ev.e1) != hipSuccess) return GX_ERR_LAUNCH;
  *gbytes_per_s = 2.0 * (double)bytes * launches / ((double)ms * 1e-3) / 1e9;
  return GX_OK;
}
