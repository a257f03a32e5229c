// HIP kernels of librmsmp for gfx950 (MI355X): row-wise mixed-scheme GEMM on int8 MFMA.
//
// All three weight classes end up as int8 operands of v_mfma_i32_16x16x64_i8:
//   4-bit Fixed codes  -> mask/shift in registers (value 16*q, undone by an exact >>4)
//   4-bit PoT codes    -> two v_perm_b32 table look-ups + xor per four codes (value +-2^(6-k))
//   8-bit Fixed codes  -> used as stored
// The FPGA design of the paper routes PoT rows to shifters and Fixed rows to multipliers
// (Section 4.1); on CDNA4 the matrix cores take int8 either way, so the scheme only decides
// how a tile is decoded.  Accumulation is int32 and exact.
#include <hip/hip_runtime.h>

#include "rmsmp_internal.h"

namespace rmsmp {

typedef int v4i __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------- operand decode

// Eight two's-complement nibbles per word -> int8 = 16*q, in MFMA slot order.
__device__ __forceinline__ v4i decode_nib_shift(uint2 w) {
  v4i a;
  a.x = (int)((w.x << 4) & 0xf0f0f0f0u);
  a.y = (int)(w.x & 0xf0f0f0f0u);
  a.z = (int)((w.y << 4) & 0xf0f0f0f0u);
  a.w = (int)(w.y & 0xf0f0f0f0u);
  return a;
}

// Four nibbles (one per byte of sel, 0..15) through the row's 16-entry byte table.
__device__ __forceinline__ uint32_t lut4(uint32_t sel, uint4 T) {
  return __builtin_amdgcn_perm(T.y, T.x, sel) ^ __builtin_amdgcn_perm(T.w, T.z, sel ^ 0x08080808u);
}

__device__ __forceinline__ v4i decode_nib_lut(uint2 w, uint4 T) {
  v4i a;
  a.x = (int)lut4(w.x & 0x0f0f0f0fu, T);
  a.y = (int)lut4((w.x >> 4) & 0x0f0f0f0fu, T);
  a.z = (int)lut4(w.y & 0x0f0f0f0fu, T);
  a.w = (int)lut4((w.y >> 4) & 0x0f0f0f0fu, T);
  return a;
}

// Sixteen unsigned 4-bit activation codes (8 bytes) -> int8 0..15 in MFMA slot order.
__device__ __forceinline__ v4i decode_act_u4(uint2 w) {
  v4i x;
  x.x = (int)(w.x & 0x0f0f0f0fu);
  x.y = (int)((w.x >> 4) & 0x0f0f0f0fu);
  x.z = (int)(w.y & 0x0f0f0f0fu);
  x.w = (int)((w.y >> 4) & 0x0f0f0f0fu);
  return x;
}

// Sixteen int8 activation codes in memory order -> MFMA slot order (even elements, then odd).
__device__ __forceinline__ v4i reorder_act_i8(uint4 w) {
  v4i x;
  x.x = (int)__builtin_amdgcn_perm(w.y, w.x, 0x06040200u);
  x.y = (int)__builtin_amdgcn_perm(w.y, w.x, 0x07050301u);
  x.z = (int)__builtin_amdgcn_perm(w.w, w.z, 0x06040200u);
  x.w = (int)__builtin_amdgcn_perm(w.w, w.z, 0x07050301u);
  return x;
}

// ---------------------------------------------------------------- epilogue

// acc -> zero-point correction -> per-row scale, bias, ReLU -> int32 / fp32 / 4-bit code.
// Every fp32 operation is rounded on its own so that codes are reproducible bit for bit.
__device__ __forceinline__ float dequant(int a, float m, bool has_bias, float b, bool relu) {
  float y = __fmul_rn((float)a, m);
  if (has_bias) y = __fadd_rn(y, b);
  if (relu) y = fmaxf(y, 0.0f);
  return y;
}

__device__ __forceinline__ uint32_t requant_u4(float y, float inv_s) {
  float t = rintf(__fmul_rn(y, inv_s));
  t = fminf(fmaxf(t, 0.0f), 15.0f);
  return (uint32_t)t;
}

// ---------------------------------------------------------------- GEMM, general tile kernel
//
// Work-group = 4 waves.  Wave w owns weight tile (blockIdx.y*4 + w): 16 rows, its packed codes
// come straight from global memory into registers (one coalesced 512-byte or 1-KiB read per
// K step) and are decoded there.  The 64 activation columns of the work-group are decoded once
// per K step into LDS as int8 and shared by the four waves, whatever their weight class.
constexpr int BN = 64;          // activation columns per work-group
constexpr int LDS_STRIDE = 80;  // bytes per column in LDS (64 + 16 pad)

template <int ACT_BITS, bool CONV, bool VEC>
__global__ __launch_bounds__(256) void gemm_tile_kernel(GemmArgs a) {
  __shared__ __attribute__((aligned(16))) uint8_t sB[BN * LDS_STRIDE];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int64_t n0 = (int64_t)blockIdx.x * BN;

  // ---- activation loader role: column lcol, 16-element chunk lchunk of each K step
  const int lcol = tid >> 2;
  const int lchunk = tid & 3;
  const int64_t ln = n0 + lcol;
  const bool ln_ok = ln < a.N;
  const uint8_t* X = (const uint8_t*)a.X;
  const int64_t ldx = ACT_BITS == 4 ? a.K / 2 : a.K;  // bytes per column (GEMM)
  int oh = 0, ow = 0, ob = 0, cchunks = 1;
  if (CONV) {
    const int64_t hw = (int64_t)a.OH * a.OW;
    const int64_t nn = ln_ok ? ln : 0;
    ob = (int)(nn / hw);
    const int rem = (int)(nn - (int64_t)ob * hw);
    oh = rem / a.OW;
    ow = rem - oh * a.OW;
    cchunks = a.d.C / KSTEP;
  }
  const uint32_t zfill = ACT_BITS == 4 ? 0x11111111u * (uint32_t)(a.ep.act_zero_point & 15)
                                       : 0x01010101u * (uint32_t)(a.ep.act_zero_point & 255);

  // ---- weight tile role
  const int mt = blockIdx.y * 4 + wave;
  const bool wave_on = mt < a.w.n_tiles;
  TileDesc td{};
  if (wave_on) td = a.w.tiles[mt];
  const int kind = td.kind;
  const int arow = lane & 15;
  uint4 T = make_uint4(0, 0, 0, 0);
  if (wave_on && kind == TILE_NIB_LUT) T = *(const uint4*)(a.w.p_lut + ((int64_t)mt * TILE_M + arow) * 4);
  const uint8_t* wbase = a.w.blob + td.blob_off;

  v4i acc[4];
  for (int j = 0; j < 4; ++j) acc[j] = (v4i){0, 0, 0, 0};

  const int nks = a.w.nks;
  for (int ks = 0; ks < nks; ++ks) {
    // -- stage the activation tile
    v4i xv = (v4i){0, 0, 0, 0};
    {
      const int k0 = ks * KSTEP + lchunk * 16;
      if (CONV) {
        const int tap = ks / cchunks;
        const int c0 = (ks - tap * cchunks) * KSTEP + lchunk * 16;
        const int kh = tap / a.d.KW, kw = tap - kh * a.d.KW;
        const int ih = oh * a.d.stride - a.d.pad + kh;
        const int iw = ow * a.d.stride - a.d.pad + kw;
        const bool inside = ln_ok && ih >= 0 && ih < a.d.H && iw >= 0 && iw < a.d.W;
        if (ACT_BITS == 4) {
          uint2 w = make_uint2(zfill, zfill);
          if (inside) w = *(const uint2*)(X + (((int64_t)ob * a.d.H + ih) * a.d.W + iw) * (a.d.C / 2) + c0 / 2);
          xv = decode_act_u4(w);
        } else {
          uint4 w = make_uint4(zfill, zfill, zfill, zfill);
          if (inside) w = *(const uint4*)(X + (((int64_t)ob * a.d.H + ih) * a.d.W + iw) * a.d.C + c0);
          xv = reorder_act_i8(w);
        }
      } else if (ACT_BITS == 4) {
        uint2 w = make_uint2(0, 0);
        if (VEC) {
          if (ln_ok && k0 < a.K) w = *(const uint2*)(X + ln * ldx + k0 / 2);
        } else if (ln_ok) {
          uint32_t b[8];
          for (int i = 0; i < 8; ++i) b[i] = (k0 + 2 * i < a.K) ? X[ln * ldx + k0 / 2 + i] : 0u;
          w.x = b[0] | (b[1] << 8) | (b[2] << 16) | (b[3] << 24);
          w.y = b[4] | (b[5] << 8) | (b[6] << 16) | (b[7] << 24);
        }
        xv = decode_act_u4(w);
      } else {
        uint4 w = make_uint4(0, 0, 0, 0);
        if (VEC) {
          if (ln_ok && k0 < a.K) w = *(const uint4*)(X + ln * ldx + k0);
        } else if (ln_ok) {
          uint32_t b[16];
          for (int i = 0; i < 16; ++i) b[i] = (k0 + i < a.K) ? X[ln * ldx + k0 + i] : 0u;
          w.x = b[0] | (b[1] << 8) | (b[2] << 16) | (b[3] << 24);
          w.y = b[4] | (b[5] << 8) | (b[6] << 16) | (b[7] << 24);
          w.z = b[8] | (b[9] << 8) | (b[10] << 16) | (b[11] << 24);
          w.w = b[12] | (b[13] << 8) | (b[14] << 16) | (b[15] << 24);
        }
        xv = reorder_act_i8(w);
      }
    }
    // -- this wave's weight fragment
    v4i av = (v4i){0, 0, 0, 0};
    if (wave_on) {
      if (kind == TILE_I8) {
        const uint4 w = *(const uint4*)(wbase + ((int64_t)ks * LANES + lane) * 16);
        av = (v4i){(int)w.x, (int)w.y, (int)w.z, (int)w.w};
      } else {
        const uint2 w = *(const uint2*)(wbase + ((int64_t)ks * LANES + lane) * 8);
        av = kind == TILE_NIB_SHIFT ? decode_nib_shift(w) : decode_nib_lut(w, T);
      }
    }
    __syncthreads();  // previous step's readers are done
    *(v4i*)(sB + lcol * LDS_STRIDE + lchunk * 16) = xv;
    __syncthreads();
    if (wave_on) {
      const int c = lane & 15, g = lane >> 4;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const v4i bv = *(const v4i*)(sB + (16 * j + c) * LDS_STRIDE + g * 16);
        acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, bv, acc[j], 0, 0, 0);
      }
    }
  }

  if (!wave_on) return;

  // ---- epilogue: lane holds rows 4*g..4*g+3 of the tile for column c of each 16-column block
  const int c = lane & 15, g = lane >> 4;
  const int zp = a.ep.act_zero_point;
  const bool has_bias = a.ep.bias != nullptr;
  const bool relu = a.ep.relu != 0;
  int orig[4], gpos[4], rsum[4];
  float m[4], bias[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int64_t p = (int64_t)mt * TILE_M + 4 * g + r;
    orig[r] = a.w.p_orig[p];
    gpos[r] = a.w.p_gpos[p];
    rsum[r] = a.w.p_rowsum[p];
    m[r] = __fmul_rn(a.w.p_rowscale[p], a.ep.act_scale);
    bias[r] = (has_bias && orig[r] >= 0) ? a.ep.bias[orig[r]] : 0.0f;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t n = n0 + 16 * j + c;
    if (n >= a.N) continue;
    int v[4] = {acc[j].x, acc[j].y, acc[j].z, acc[j].w};
    uint32_t q[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (kind == TILE_NIB_SHIFT) v[r] >>= 4;
      v[r] -= zp * rsum[r];
      if (a.ep.out_kind == 0) {
        if (orig[r] >= 0) ((int32_t*)a.Y)[(int64_t)orig[r] * a.N + n] = v[r];
      } else {
        const float y = dequant(v[r], m[r], has_bias, bias[r], relu);
        if (a.ep.out_kind == 1) {
          if (orig[r] >= 0) ((float*)a.Y)[(int64_t)orig[r] * a.N + n] = y;
        } else {
          q[r] = requant_u4(y, a.ep.out_inv_scale);
        }
      }
    }
    if (a.ep.out_kind == 2) {
      uint8_t* Yb = (uint8_t*)a.Y + n * (a.M / 2);
      if (gpos[0] >= 0) Yb[gpos[0] >> 1] = (uint8_t)(q[0] | (q[1] << 4));
      if (gpos[2] >= 0) Yb[gpos[2] >> 1] = (uint8_t)(q[2] | (q[3] << 4));
    }
  }
}

template <int ACT_BITS, bool CONV, bool VEC>
static int launch_one(const GemmArgs& a, hipStream_t s) {
  dim3 grid((unsigned)((a.N + BN - 1) / BN), (unsigned)((a.w.n_tiles + 3) / 4), 1);
  hipLaunchKernelGGL((gemm_tile_kernel<ACT_BITS, CONV, VEC>), grid, dim3(256), 0, s, a);
  return (int)hipGetLastError();
}

int launch_gemm(const GemmArgs& a, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  if (a.N <= 0) return 0;
  if (a.conv) {
    return a.ep.act_bits == 4 ? launch_one<4, true, true>(a, s) : launch_one<8, true, true>(a, s);
  }
  const bool vec = (a.K % 16) == 0;
  if (a.ep.act_bits == 4) return vec ? launch_one<4, false, true>(a, s) : launch_one<4, false, false>(a, s);
  return vec ? launch_one<8, false, true>(a, s) : launch_one<8, false, false>(a, s);
}

// ---------------------------------------------------------------- explicit im2col
//
// Fallback for layers whose channel count is not a multiple of the K step: writes the lowered
// matrix [N][Kpad] in the K order the weights are stored in, (kh, kw) outer and channel inner.
// One thread per output byte.
template <int ACT_BITS>
__global__ __launch_bounds__(256) void im2col_kernel(Im2colArgs a) {
  const int64_t row_bytes = ACT_BITS == 4 ? a.Kpad / 2 : a.Kpad;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= a.N * row_bytes) return;
  const int64_t n = idx / row_bytes;
  const int64_t bofs = idx - n * row_bytes;
  const int64_t hw = (int64_t)a.OH * a.OW;
  const int b = (int)(n / hw);
  const int rem = (int)(n - (int64_t)b * hw);
  const int oh = rem / a.OW, ow = rem - oh * a.OW;
  const uint8_t* X = (const uint8_t*)a.X;
  auto code = [&](int64_t kk) -> uint32_t {
    if (kk >= a.K) return 0u;
    const int tap = (int)(kk / a.d.C), cc = (int)(kk - (int64_t)tap * a.d.C);
    const int kh = tap / a.d.KW, kw = tap - kh * a.d.KW;
    const int ih = oh * a.d.stride - a.d.pad + kh, iw = ow * a.d.stride - a.d.pad + kw;
    if (ih < 0 || ih >= a.d.H || iw < 0 || iw >= a.d.W) return (uint32_t)a.zero_point & (ACT_BITS == 4 ? 15u : 255u);
    const int64_t pix = ((int64_t)b * a.d.H + ih) * a.d.W + iw;
    if (ACT_BITS == 4) {
      const uint32_t byte = X[pix * (a.d.C / 2) + cc / 2];
      return (cc & 1) ? (byte >> 4) : (byte & 15u);
    }
    return X[pix * a.d.C + cc];
  };
  uint8_t* out = (uint8_t*)a.cols;
  if (ACT_BITS == 4) {
    out[idx] = (uint8_t)(code(2 * bofs) | (code(2 * bofs + 1) << 4));
  } else {
    out[idx] = (uint8_t)code(bofs);
  }
}

int launch_im2col(const Im2colArgs& a, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  const int64_t row_bytes = a.act_bits == 4 ? a.Kpad / 2 : a.Kpad;
  const int64_t total = a.N * row_bytes;
  if (total <= 0) return 0;
  dim3 grid((unsigned)((total + 255) / 256));
  if (a.act_bits == 4)
    hipLaunchKernelGGL(im2col_kernel<4>, grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(im2col_kernel<8>, grid, dim3(256), 0, s, a);
  return (int)hipGetLastError();
}

}  // namespace rmsmp
