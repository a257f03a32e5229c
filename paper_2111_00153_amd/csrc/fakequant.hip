// Quantization-aware-training helpers: the weight side of Alg. 1's loop body on the device.
//   forward   What = proj_S(W): every row projected onto the level set of its own scheme with its
//             own scaling factor (Eq. 1-4), written back as fp32 = rowscale * integer level --
//             bit for bit the value the packed inference path multiplies with;
//   backward  the straight-through estimator (Eq. 5): dW = dWhat, zero where the clip was active.
// Both are streaming kernels bound by HBM (8 bytes per weight for the forward: one read that
// misses, one write; the second read of a row hits in L2).  gfx950 only.
#include <hip/hip_runtime.h>

#include "rmsmp_internal.h"

namespace rmsmp {

namespace {

constexpr int FQ_THREADS = 256;

// w/alpha limited to [-1, 1] (the clip of Section 3.1.1), one correctly rounded divide.
__device__ __forceinline__ float clip_ratio(float w, float alpha) {
  if (w < -alpha) return -1.0f;
  if (w > alpha) return 1.0f;
  return __fdiv_rn(w, alpha);
}

// Fixed-m level of x in [-1, 1] as an integer in [-Q, Q], round half to even (Eq. 1-2).
__device__ __forceinline__ int fixed_int(float x, float Q) { return (int)rintf(__fmul_rn(x, Q)); }

// PoT-4 level of x in [-1, 1] as sign * 2^(6-k), k = 0..6, or 0 (Eq. 3-4).  The base-2 logarithm
// is rounded exactly: |x| = f * 2^e with f in [1, 2) rounds up iff f > sqrt(2), and the largest
// float below sqrt(2) has the fraction bits 0x3504f3.
__device__ __forceinline__ int pot4_int(float x) {
  const float a = fabsf(x);
  if (!(a > 0.0078125f)) return 0;  // at or below half of the smallest level, 2^-7
  const uint32_t bits = __float_as_uint(a);
  int e = (int)(bits >> 23) - 127;
  if ((bits & 0x7fffffu) > 0x3504f3u) e += 1;
  e = e > 0 ? 0 : e < -6 ? -6 : e;
  const int mag = 1 << (6 + e);
  return x < 0.0f ? -mag : mag;
}

__device__ __forceinline__ float project_one(float w, float alpha, int scheme, float rowscale, float Q) {
  const float x = clip_ratio(w, alpha);
  const int q = scheme == RMSMP_POT4 ? pot4_int(x) : fixed_int(x, Q);
  return __fmul_rn(rowscale, (float)q);
}

// max over the work-group; every thread gets the result
__device__ __forceinline__ float block_max(float v, float* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  float m = red[0];
#pragma unroll
  for (int i = 1; i < FQ_THREADS / 64; ++i) m = fmaxf(m, red[i]);
  return m;
}

// Rows of up to FQ_CACHED_K weights (16-byte aligned, K % 4 == 0) with no alpha supplied: the row
// is read once, kept in registers while its maximum is found, then projected and written.
constexpr int FQ_CACHED_VEC = 8;                                // float4 per thread
constexpr int64_t FQ_CACHED_K = (int64_t)FQ_THREADS * FQ_CACHED_VEC * 4;  // 8192

__global__ __launch_bounds__(FQ_THREADS) void fake_quant_rows_cached_kernel(FakeQuantArgs a) {
  __shared__ float red[FQ_THREADS / 64];
  const int64_t r = blockIdx.x;
  const float4* w4 = (const float4*)(a.W + r * a.K);
  float4* o4 = (float4*)(a.What + r * a.K);
  const int tid = threadIdx.x;
  const int n4 = (int)(a.K / 4);
  float4 v[FQ_CACHED_VEC];
  float m = 0.0f;
#pragma unroll
  for (int j = 0; j < FQ_CACHED_VEC; ++j) {
    const int i = tid + j * FQ_THREADS;
    v[j] = i < n4 ? w4[i] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    m = fmaxf(m, fmaxf(fmaxf(fabsf(v[j].x), fabsf(v[j].y)), fmaxf(fabsf(v[j].z), fabsf(v[j].w))));
  }
  float alpha = block_max(m, red);
  if (alpha == 0.0f) alpha = 1.0f;
  if (a.alpha_out && tid == 0) a.alpha_out[r] = alpha;
  const int scheme = a.scheme[r];
  const float Q = scheme == RMSMP_FIXED4 ? 7.0f : 127.0f;
  const float rowscale = scheme == RMSMP_POT4 ? __fmul_rn(alpha, 0.015625f) : __fdiv_rn(alpha, Q);
#pragma unroll
  for (int j = 0; j < FQ_CACHED_VEC; ++j) {
    const int i = tid + j * FQ_THREADS;
    if (i >= n4) continue;
    float4 o;
    o.x = project_one(v[j].x, alpha, scheme, rowscale, Q);
    o.y = project_one(v[j].y, alpha, scheme, rowscale, Q);
    o.z = project_one(v[j].z, alpha, scheme, rowscale, Q);
    o.w = project_one(v[j].w, alpha, scheme, rowscale, Q);
    o4[i] = o;
  }
}

// One work-group per row, any K.  VEC: rows are 16-byte aligned and K % 4 == 0.
template <bool VEC>
__global__ __launch_bounds__(FQ_THREADS) void fake_quant_rows_kernel(FakeQuantArgs a) {
  __shared__ float red[FQ_THREADS / 64];
  const int64_t r = blockIdx.x;
  const float* w = a.W + r * a.K;
  float* out = a.What + r * a.K;
  const int tid = threadIdx.x;
  float alpha;
  if (a.alpha) {
    alpha = a.alpha[r];
  } else {
    float m = 0.0f;
    if (VEC) {
      const float4* w4 = (const float4*)w;
      for (int64_t i = tid; i < a.K / 4; i += FQ_THREADS) {
        const float4 v = w4[i];
        m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
      }
    } else {
      for (int64_t i = tid; i < a.K; i += FQ_THREADS) m = fmaxf(m, fabsf(w[i]));
    }
    alpha = block_max(m, red);
    if (alpha == 0.0f) alpha = 1.0f;
  }
  if (a.alpha_out && tid == 0) a.alpha_out[r] = alpha;
  const int scheme = a.scheme[r];
  const float Q = scheme == RMSMP_FIXED4 ? 7.0f : 127.0f;
  const float rowscale = scheme == RMSMP_POT4 ? __fmul_rn(alpha, 0.015625f) : __fdiv_rn(alpha, Q);
  if (VEC) {
    const float4* w4 = (const float4*)w;
    float4* o4 = (float4*)out;
    for (int64_t i = tid; i < a.K / 4; i += FQ_THREADS) {
      const float4 v = w4[i];
      float4 o;
      o.x = project_one(v.x, alpha, scheme, rowscale, Q);
      o.y = project_one(v.y, alpha, scheme, rowscale, Q);
      o.z = project_one(v.z, alpha, scheme, rowscale, Q);
      o.w = project_one(v.w, alpha, scheme, rowscale, Q);
      o4[i] = o;
    }
  } else {
    for (int64_t i = tid; i < a.K; i += FQ_THREADS) out[i] = project_one(w[i], alpha, scheme, rowscale, Q);
  }
}

template <bool VEC>
__global__ __launch_bounds__(FQ_THREADS) void ste_backward_kernel(SteArgs a) {
  const int64_t r = blockIdx.x;
  const float* g = a.dWhat + r * a.K;
  float* out = a.dW + r * a.K;
  const int tid = threadIdx.x;
  if (!a.alpha) {  // nothing was clipped: the gradient passes unchanged
    if (VEC) {
      for (int64_t i = tid; i < a.K / 4; i += FQ_THREADS) ((float4*)out)[i] = ((const float4*)g)[i];
    } else {
      for (int64_t i = tid; i < a.K; i += FQ_THREADS) out[i] = g[i];
    }
    return;
  }
  const float alpha = a.alpha[r];
  const float* w = a.W + r * a.K;
  if (VEC) {
    for (int64_t i = tid; i < a.K / 4; i += FQ_THREADS) {
      const float4 v = ((const float4*)w)[i];
      float4 o = ((const float4*)g)[i];
      o.x = fabsf(v.x) > alpha ? 0.0f : o.x;
      o.y = fabsf(v.y) > alpha ? 0.0f : o.y;
      o.z = fabsf(v.z) > alpha ? 0.0f : o.z;
      o.w = fabsf(v.w) > alpha ? 0.0f : o.w;
      ((float4*)out)[i] = o;
    }
  } else {
    for (int64_t i = tid; i < a.K; i += FQ_THREADS) out[i] = fabsf(w[i]) > alpha ? 0.0f : g[i];
  }
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

int launch_fake_quant_rows(const FakeQuantArgs& a, void* stream) {
  if (a.M <= 0 || a.K <= 0) return 0;
  const bool vec = a.K % 4 == 0 && aligned16(a.W) && aligned16(a.What);
  const dim3 grid((unsigned)a.M), block(FQ_THREADS);
  if (vec && !a.alpha && a.K <= FQ_CACHED_K)
    hipLaunchKernelGGL(fake_quant_rows_cached_kernel, grid, block, 0, (hipStream_t)stream, a);
  else if (vec)
    hipLaunchKernelGGL(fake_quant_rows_kernel<true>, grid, block, 0, (hipStream_t)stream, a);
  else
    hipLaunchKernelGGL(fake_quant_rows_kernel<false>, grid, block, 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

int launch_ste_backward(const SteArgs& a, void* stream) {
  if (a.M <= 0 || a.K <= 0) return 0;
  const bool vec = a.K % 4 == 0 && aligned16(a.dWhat) && aligned16(a.dW) && (!a.alpha || aligned16(a.W));
  const dim3 grid((unsigned)a.M), block(FQ_THREADS);
  if (vec)
    hipLaunchKernelGGL(ste_backward_kernel<true>, grid, block, 0, (hipStream_t)stream, a);
  else
    hipLaunchKernelGGL(ste_backward_kernel<false>, grid, block, 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

}  // namespace rmsmp
