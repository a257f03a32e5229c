// Two machine-rate measurements behind rmsmp_debug_measure_peaks: what this GPU sustains with
// nothing but int8 MFMAs in flight, and with nothing but a copy.  Benchmarks quote them next to
// the published peaks so that a kernel's fraction can be read against either.
#include <hip/hip_runtime.h>

#include "device_common.h"

namespace rmsmp {

// Two waves per SIMD, each with eight independent 32x32 accumulators and operands that never
// leave registers: the matrix pipe is the only unit with work.
__global__ __launch_bounds__(512) void mfma_only_kernel(int* sink, int iters) {
  const int lane = threadIdx.x & 63;
  v16i acc[8];
#pragma unroll
  for (int m = 0; m < 8; ++m)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[m][r] = 0;
  const v4i a = {lane, lane + 1, lane + 2, lane + 3}, b = {1, 2, 3, 4};
#pragma unroll 1
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 8; ++m) acc[m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[m], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int m = 0; m < 8; ++m)
#pragma unroll
    for (int r = 0; r < 16; ++r) s ^= acc[m][r];
  if (s == 0x7fffffff) sink[0] = s;  // keeps the accumulators alive; practically never taken
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  // four independent 16-byte loads in flight per thread
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a, dst[i + stride] = b, dst[i + 2 * stride] = c, dst[i + 3 * stride] = d;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

// Returns hipError_t as int.  Allocates and frees 2 GiB of device memory; synchronizes.
int measure_peaks(double* mfma_tops, double* copy_gbs) {
  hipError_t e;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  void *src = nullptr, *dst = nullptr;
  int* sink = nullptr;
  const size_t bytes = (size_t)1 << 30;
  float ms = 0.0f;
  auto done = [&](hipError_t rc) {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (src) (void)hipFree(src);
    if (dst) (void)hipFree(dst);
    if (sink) (void)hipFree(sink);
    return (int)rc;
  };
  if ((e = hipEventCreate(&e0)) != hipSuccess) return done(e);
  if ((e = hipEventCreate(&e1)) != hipSuccess) return done(e);
  if ((e = hipMalloc((void**)&sink, 256)) != hipSuccess) return done(e);
  hipDeviceProp_t prop;
  int dev = 0;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return done(e);
  if ((e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return done(e);
  const int cus = prop.multiProcessorCount;
  // ---- MFMA only
  const int iters = 4000;
  hipLaunchKernelGGL(mfma_only_kernel, dim3(cus), dim3(512), 0, 0, sink, 200);  // warm-up
  if ((e = hipEventRecord(e0, 0)) != hipSuccess) return done(e);
  hipLaunchKernelGGL(mfma_only_kernel, dim3(cus), dim3(512), 0, 0, sink, iters);
  if ((e = hipEventRecord(e1, 0)) != hipSuccess) return done(e);
  if ((e = hipEventSynchronize(e1)) != hipSuccess) return done(e);
  if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) return done(e);
  if (mfma_tops) *mfma_tops = (double)cus * 8 /*waves*/ * iters * 8 /*MFMAs*/ * (2.0 * 32 * 32 * 32) / (ms * 1e-3) / 1e12;
  // ---- copy
  if ((e = hipMalloc(&src, bytes)) != hipSuccess) return done(e);
  if ((e = hipMalloc(&dst, bytes)) != hipSuccess) return done(e);
  if ((e = hipMemset(src, 1, bytes)) != hipSuccess) return done(e);
  if ((e = hipMemset(dst, 0, bytes)) != hipSuccess) return done(e);
  hipLaunchKernelGGL(stream_copy_kernel, dim3(cus * 8), dim3(256), 0, 0, (const uint4*)src, (uint4*)dst, bytes / 16);
  if ((e = hipEventRecord(e0, 0)) != hipSuccess) return done(e);
  for (int r = 0; r < 5; ++r)
    hipLaunchKernelGGL(stream_copy_kernel, dim3(cus * 8), dim3(256), 0, 0, (const uint4*)src, (uint4*)dst, bytes / 16);
  if ((e = hipEventRecord(e1, 0)) != hipSuccess) return done(e);
  if ((e = hipEventSynchronize(e1)) != hipSuccess) return done(e);
  if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) return done(e);
  if (copy_gbs) *copy_gbs = 5.0 * 2.0 * (double)bytes / (ms * 1e-3) / 1e9;
  return done(hipGetLastError());
}

}  // namespace rmsmp
