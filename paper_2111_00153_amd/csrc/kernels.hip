// HIP kernels of librmsmp for gfx950 (MI355X): row-wise mixed-scheme GEMM on int8 MFMA.
//
// All three weight classes end up as int8 operands of v_mfma_i32_32x32x32_i8:
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
typedef int v16i __attribute__((ext_vector_type(16)));

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

// Packed weight fragment of one K step as it sits in memory (per lane): 8 bytes of nibbles or
// 16 bytes of int8.
template <int KIND>
struct RawFrag {
  typedef uint2 type;
};
template <>
struct RawFrag<TILE_I8> {
  typedef uint4 type;
};

template <int KIND>
__device__ __forceinline__ typename RawFrag<KIND>::type load_raw(const uint8_t* lane_ptr, int64_t step_bytes_index) {
  return *(const typename RawFrag<KIND>::type*)(lane_ptr + step_bytes_index);
}

template <int KIND>
__device__ __forceinline__ v4i decode_raw(typename RawFrag<KIND>::type w, uint4 T);
template <>
__device__ __forceinline__ v4i decode_raw<TILE_NIB_SHIFT>(uint2 w, uint4) {
  return decode_nib_shift(w);
}
template <>
__device__ __forceinline__ v4i decode_raw<TILE_NIB_LUT>(uint2 w, uint4 T) {
  return decode_nib_lut(w, T);
}
template <>
__device__ __forceinline__ v4i decode_raw<TILE_I8>(uint4 w, uint4) {
  return (v4i){(int)w.x, (int)w.y, (int)w.z, (int)w.w};
}

// ---------------------------------------------------------------- epilogue

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

// Row metadata of the 16 grouped rows a lane finishes: {rowscale bits, rowsum, original row, grouped position}.
struct RowMeta {
  int4 m[16];
};

__device__ __forceinline__ void load_row_meta(const GemmArgs& a, int mt, int lane, RowMeta& rm) {
  const int4* src = (const int4*)a.w.p_meta + (int64_t)mt * TILE_M + 16 * (lane >> 5);
#pragma unroll
  for (int r = 0; r < 16; ++r) rm.m[r] = src[r];
}

// Finish one 32x32 accumulator tile: zero-point correction, per-row scale, bias, ReLU, then
// int32 / fp32 / nibble-packed 4-bit store.  Register r of lane l is grouped row 16*(l/32)+r of
// the weight tile and column n; the 16 registers of a lane are 16 consecutive grouped rows.
__device__ __forceinline__ void finish_tile(const GemmArgs& a, int kind, const v16i& acc, const RowMeta& rm,
                                            int64_t n) {
  if (n >= a.N) return;
  const int zp = a.ep.act_zero_point;
  const bool has_bias = a.ep.bias != nullptr;
  const bool relu = a.ep.relu != 0;
  const int out_kind = a.ep.out_kind;
  uint32_t packed[2] = {0u, 0u};
  int n_rows = 0;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int orig = rm.m[r].z;
    if (orig < 0) continue;
    ++n_rows;
    int v = acc[r];
    if (kind == TILE_NIB_SHIFT) v >>= 4;
    v -= zp * rm.m[r].y;
    if (out_kind == 0) {
      ((int32_t*)a.Y)[(int64_t)orig * a.N + n] = v;
    } else {
      const float m = __fmul_rn(__int_as_float(rm.m[r].x), a.ep.act_scale);
      const float y = dequant(v, m, has_bias, has_bias ? a.ep.bias[orig] : 0.0f, relu);
      if (out_kind == 1) {
        ((float*)a.Y)[(int64_t)orig * a.N + n] = y;
      } else {
        packed[r >> 3] |= requant_u4(y, a.ep.out_inv_scale) << (4 * (r & 7));
      }
    }
  }
  if (out_kind == 2 && n_rows > 0) {
    // valid rows of a tile are a prefix, so they start at register 0 and the first grouped
    // position is a multiple of 16
    uint8_t* dst = (uint8_t*)a.Y + n * (a.M / 2) + (rm.m[0].w >> 1);
    if (n_rows == 16 && (((uintptr_t)dst) & 7) == 0) {
      *(uint2*)dst = make_uint2(packed[0], packed[1]);
    } else {
      for (int b = 0; b < n_rows / 2; ++b) dst[b] = (uint8_t)(packed[b >> 2] >> (8 * (b & 3)));
    }
  }
}

// ---------------------------------------------------------------- general tile kernel
//
// Work-group = 4 waves.  Wave w owns weight tile (blockIdx.y*4 + w): 32 rows, its packed codes
// come straight from global memory into registers (one coalesced 512-byte or 1-KiB read per
// K step) and are decoded there.  The 64 activation columns of the work-group are decoded once
// per 64-deep K slab into LDS as int8 and shared by the four waves, whatever their weight class.
// Handles every shape: plain GEMM, implicit im2col for any stride / padding (C % 16 == 0).
constexpr int GEN_BN = 64;      // activation columns per work-group
constexpr int GEN_BK = 64;      // K elements staged per step
constexpr int GEN_STRIDE = 80;  // bytes per column in LDS (64 + 16 pad)

template <int KIND>
__device__ __forceinline__ void general_slab_mfma(const uint8_t* lane_ptr, int s, uint4 T, const uint8_t* sB, int lane,
                                                  v16i (&acc)[2], typename RawFrag<KIND>::type w0,
                                                  typename RawFrag<KIND>::type w1) {
  const v4i av0 = decode_raw<KIND>(w0, T);
  const v4i av1 = decode_raw<KIND>(w1, T);
  const int c = lane & 31, kb = lane >> 5;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const v4i b0 = *(const v4i*)(sB + (32 * j + c) * GEN_STRIDE + kb * 16);
    const v4i b1 = *(const v4i*)(sB + (32 * j + c) * GEN_STRIDE + 32 + kb * 16);
    acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av0, b0, acc[j], 0, 0, 0);
    acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av1, b1, acc[j], 0, 0, 0);
  }
}

template <int ACT_BITS, bool CONV, bool VEC>
__global__ __launch_bounds__(256) void gemm_general_kernel(GemmArgs a) {
  __shared__ __attribute__((aligned(16))) uint8_t sB[GEN_BN * GEN_STRIDE];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t n0 = (int64_t)blockIdx.x * GEN_BN;

  // ---- activation loader role: column lcol, 16-element chunk lchunk of each K slab
  const int lcol = tid >> 2;
  const int lchunk = tid & 3;
  const int64_t ln = n0 + lcol;
  const bool ln_ok = ln < a.N;
  const uint8_t* X = (const uint8_t*)a.X;
  const int64_t ldx = ACT_BITS == 4 ? a.K / 2 : a.K;  // bytes per column (GEMM)
  int oh = 0, ow = 0, ob = 0;
  if (CONV) {
    const int64_t hw = (int64_t)a.OH * a.OW;
    const int64_t nn = ln_ok ? ln : 0;
    ob = (int)(nn / hw);
    const int rem = (int)(nn - (int64_t)ob * hw);
    oh = rem / a.OW;
    ow = rem - oh * a.OW;
  }
  const uint32_t zfill = ACT_BITS == 4 ? 0x11111111u * (uint32_t)(a.ep.act_zero_point & 15)
                                       : 0x01010101u * (uint32_t)(a.ep.act_zero_point & 255);

  // ---- weight tile role
  const int mt = blockIdx.y * 4 + wave;
  const bool wave_on = mt < a.w.n_tiles;
  int kind = TILE_NIB_SHIFT;
  int64_t blob_off = 0;
  if (wave_on) {
    kind = __builtin_amdgcn_readfirstlane(a.w.tiles[mt].kind);
    blob_off = a.w.tiles[mt].blob_off;
  }
  uint4 T = make_uint4(0, 0, 0, 0);
  if (wave_on && kind == TILE_NIB_LUT)
    T = *(const uint4*)(a.w.p_lut + ((int64_t)mt * TILE_M + tile_row_goff(lane & 31)) * 4);
  const int frag_bytes = kind == TILE_I8 ? 16 : 8;
  const uint8_t* lane_ptr = a.w.blob + blob_off + (int64_t)lane * frag_bytes;
  const int64_t step_bytes = (int64_t)LANES * frag_bytes;

  v16i acc[2];
  for (int j = 0; j < 2; ++j)
    for (int r = 0; r < 16; ++r) acc[j][r] = 0;

  const int nslab = a.w.nks / 2;
  for (int s = 0; s < nslab; ++s) {
    // -- stage the activation slab
    v4i xv = (v4i){0, 0, 0, 0};
    {
      const int k0 = s * GEN_BK + lchunk * 16;
      if (CONV) {
        const int tap = k0 / a.d.C;
        const int c0 = k0 - tap * a.d.C;
        const int kh = tap / a.d.KW, kw = tap - kh * a.d.KW;
        const int ih = oh * a.d.stride - a.d.pad + kh;
        const int iw = ow * a.d.stride - a.d.pad + kw;
        const bool live = ln_ok && k0 < a.K;
        const bool inside = live && ih >= 0 && ih < a.d.H && iw >= 0 && iw < a.d.W;
        if (ACT_BITS == 4) {
          uint2 w = live ? make_uint2(zfill, zfill) : make_uint2(0, 0);
          if (inside) w = *(const uint2*)(X + (((int64_t)ob * a.d.H + ih) * a.d.W + iw) * (a.d.C / 2) + c0 / 2);
          xv = decode_act_u4(w);
        } else {
          uint4 w = live ? make_uint4(zfill, zfill, zfill, zfill) : make_uint4(0, 0, 0, 0);
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
    // -- this wave's two packed weight fragments of the slab (decoded after the barrier)
    uint4 raw0 = make_uint4(0, 0, 0, 0), raw1 = raw0;
    if (wave_on) {
      if (kind == TILE_I8) {
        raw0 = load_raw<TILE_I8>(lane_ptr, (2 * s) * step_bytes);
        raw1 = load_raw<TILE_I8>(lane_ptr, (2 * s + 1) * step_bytes);
      } else {
        const uint2 w0 = load_raw<TILE_NIB_SHIFT>(lane_ptr, (2 * s) * step_bytes);
        const uint2 w1 = load_raw<TILE_NIB_SHIFT>(lane_ptr, (2 * s + 1) * step_bytes);
        raw0 = make_uint4(w0.x, w0.y, 0, 0);
        raw1 = make_uint4(w1.x, w1.y, 0, 0);
      }
    }
    __syncthreads();  // previous slab's readers are done
    *(v4i*)(sB + lcol * GEN_STRIDE + lchunk * 16) = xv;
    __syncthreads();
    if (wave_on) {
      if (kind == TILE_NIB_SHIFT)
        general_slab_mfma<TILE_NIB_SHIFT>(lane_ptr, s, T, sB, lane, acc, make_uint2(raw0.x, raw0.y),
                                          make_uint2(raw1.x, raw1.y));
      else if (kind == TILE_NIB_LUT)
        general_slab_mfma<TILE_NIB_LUT>(lane_ptr, s, T, sB, lane, acc, make_uint2(raw0.x, raw0.y),
                                        make_uint2(raw1.x, raw1.y));
      else
        general_slab_mfma<TILE_I8>(lane_ptr, s, T, sB, lane, acc, raw0, raw1);
    }
  }

  if (!wave_on) return;
  RowMeta rm;
  load_row_meta(a, mt, lane, rm);
#pragma unroll
  for (int j = 0; j < 2; ++j) finish_tile(a, kind, acc[j], rm, n0 + 32 * j + (lane & 31));
}

template <int ACT_BITS, bool CONV, bool VEC>
static int launch_general(const GemmArgs& a, hipStream_t s) {
  dim3 grid((unsigned)((a.N + GEN_BN - 1) / GEN_BN), (unsigned)((a.w.n_tiles + 3) / 4), 1);
  hipLaunchKernelGGL((gemm_general_kernel<ACT_BITS, CONV, VEC>), grid, dim3(256), 0, s, a);
  return (int)hipGetLastError();
}

// ---------------------------------------------------------------- stride-1 convolution kernel
//
// Implicit im2col with the input patch resident in LDS.  A work-group produces 64 output rows
// (two weight tiles) x 128 output pixels.  The pixels it needs -- a contiguous run of the
// flattened NHWC input -- are read from memory once, decoded to int8 and kept in LDS for all
// KH*KW taps; out-of-image taps point at a row filled with the zero-point code.  The patch is
// shared by both weight tiles whatever their class.  Eight waves: each pair of waves owns one
// weight tile x 64 pixels and splits the K steps between them (even / odd), so that one wave's
// decode and LDS reads run under the other's MFMAs (a wave cannot overlap its own); the two
// partial sums are added through LDS at the end (int32 addition is exact in any order).
// Packed weights stream from global memory straight into a register ring that runs PT_RING K
// steps ahead of the MFMAs; everything is unrolled so that the ring is addressed statically.
constexpr int PT_BN = 128;

template <int KIND, int TAPS, int CPT>
__device__ __forceinline__ void patch_mainloop(const uint8_t* lane_ptr, uint4 T, const uint8_t* smem,
                                               const int (&row_addr)[2], const uint32_t (&vmask)[2], int zaddr,
                                               int tap_row_bytes, int tap_col_bytes, v16i (&acc)[2]) {
  constexpr int OWN_PER_TAP = CPT / 2;
  constexpr int NOWN = TAPS * OWN_PER_TAP;
  constexpr int FRAG = KIND == TILE_I8 ? 16 : 8;
  constexpr int RING = NOWN < (KIND == TILE_I8 ? 12 : 18) ? NOWN : (KIND == TILE_I8 ? 12 : 18);
  constexpr int64_t OWN_STRIDE = 2 * LANES * FRAG;  // this wave takes every other K step
  typename RawFrag<KIND>::type ring[RING];
#pragma unroll
  for (int u = 0; u < RING; ++u) ring[u] = load_raw<KIND>(lane_ptr, u * OWN_STRIDE);
  // LDS address of this lane's B fragment for every tap and both pixel blocks
  constexpr int KW3 = TAPS == 9 ? 3 : 1;
  int addr[TAPS][2];
#pragma unroll
  for (int t = 0; t < TAPS; ++t) {
    const int toff = (t / KW3) * tap_row_bytes + (t % KW3) * tap_col_bytes;
#pragma unroll
    for (int j = 0; j < 2; ++j) addr[t][j] = ((vmask[j] >> t) & 1u) ? row_addr[j] + toff : zaddr;
  }
  // B fragments are read one step ahead of the MFMAs that use them
  v4i b0 = *(const v4i*)(smem + addr[0][0]);
  v4i b1 = *(const v4i*)(smem + addr[0][1]);
#pragma unroll
  for (int s = 0; s < NOWN; ++s) {
    const v4i av = decode_raw<KIND>(ring[s % RING], T);
    if (s + RING < NOWN) ring[s % RING] = load_raw<KIND>(lane_ptr, (int64_t)(s + RING) * OWN_STRIDE);
    v4i nb0 = b0, nb1 = b1;
    if (s + 1 < NOWN) {
      const int t1 = (s + 1) / OWN_PER_TAP, u1 = (s + 1) % OWN_PER_TAP;
      nb0 = *(const v4i*)(smem + addr[t1][0] + u1 * 2 * KSTEP);
      nb1 = *(const v4i*)(smem + addr[t1][1] + u1 * 2 * KSTEP);
    }
    acc[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, b0, acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, b1, acc[1], 0, 0, 0);
    b0 = nb0;
    b1 = nb1;
    // keep each step's prefetch where it is: without this the scheduler sinks the loads next
    // to their use and the ring degenerates to one or two loads in flight
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int TAPS, int CPT>
__global__ __launch_bounds__(512) void conv_patch_kernel(GemmArgs a, int row_stride, int patch_rows) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int pair = wave & 3;     // which (weight tile, 64-pixel half)
  const int parity = wave >> 2;  // which K steps
  const int mi = pair >> 1, nh = pair & 1;
  const int64_t n0 = (int64_t)blockIdx.x * PT_BN;
  constexpr int C = CPT * KSTEP;
  constexpr int KW = TAPS == 9 ? 3 : 1;
  const int H = a.d.H, W = a.d.W, pad = a.d.pad;
  const int hw_out = a.OH * a.OW;

  // ---- weight tile of this wave pair; start its stream and the row metadata right away
  const int mt = blockIdx.y * 2 + mi;
  const bool wave_on = mt < a.w.n_tiles;
  int kind = TILE_NIB_SHIFT;
  int64_t blob_off = 0;
  if (wave_on) {
    kind = __builtin_amdgcn_readfirstlane(a.w.tiles[mt].kind);
    blob_off = a.w.tiles[mt].blob_off;
  }
  uint4 T = make_uint4(0, 0, 0, 0);
  if (wave_on && kind == TILE_NIB_LUT)
    T = *(const uint4*)(a.w.p_lut + ((int64_t)mt * TILE_M + tile_row_goff(lane & 31)) * 4);
  const int frag_bytes = kind == TILE_I8 ? 16 : 8;
  const uint8_t* lane_ptr = a.w.blob + blob_off + ((int64_t)parity * LANES + lane) * frag_bytes;

  // flattened input index of tap (0,0) for output pixel n (may be negative / out of image)
  auto base_index = [&](int64_t n, int& b, int& oh, int& ow) -> int64_t {
    b = (int)(n / hw_out);
    const int rem = (int)(n - (int64_t)b * hw_out);
    oh = rem / a.OW;
    ow = rem - oh * a.OW;
    return ((int64_t)b * H + (oh - pad)) * W + (ow - pad);
  };
  int tb, toh, tow;
  int64_t f_lo = base_index(n0, tb, toh, tow);
  if (f_lo < 0) f_lo = 0;
  const int64_t total_px = (int64_t)a.d.B * H * W;

  // ---- stage the patch: pixels f_lo .. f_lo+patch_rows-1, decoded to int8, row_stride bytes each.
  // Loads are issued in batches of PATCH_UNROLL before the first use so that they overlap.
  {
    const uint8_t* X = (const uint8_t*)a.X;
    constexpr int CHUNKS = C / 16;  // 16-channel chunks per pixel
    constexpr int PATCH_UNROLL = 6;
    const int total = patch_rows * CHUNKS;
    for (int base = 0; base < total; base += 512 * PATCH_UNROLL) {
      uint2 w[PATCH_UNROLL];
#pragma unroll
      for (int u = 0; u < PATCH_UNROLL; ++u) {
        const int idx = base + u * 512 + tid;
        const int px = idx / CHUNKS, ch = idx % CHUNKS;
        const int64_t f = f_lo + px;
        w[u] = make_uint2(0, 0);
        if (idx < total && f < total_px) w[u] = *(const uint2*)(X + f * (C / 2) + ch * 8);
      }
#pragma unroll
      for (int u = 0; u < PATCH_UNROLL; ++u) {
        const int idx = base + u * 512 + tid;
        const int px = idx / CHUNKS, ch = idx % CHUNKS;
        if (idx < total) *(v4i*)(smem + px * row_stride + ch * 16) = decode_act_u4(w[u]);
      }
    }
    // the zero-point row
    const uint32_t zf = 0x01010101u * (uint32_t)(a.ep.act_zero_point & 15);
    if (tid < CHUNKS) *(v4i*)(smem + patch_rows * row_stride + tid * 16) = (v4i){(int)zf, (int)zf, (int)zf, (int)zf};
  }

  // ---- per-lane LDS address of tap (0,0) and validity mask over the taps, for both pixel blocks
  const int lane_off = 16 * (lane >> 5) + parity * KSTEP;
  const int zaddr = patch_rows * row_stride + lane_off;
  int row_addr[2];
  uint32_t vmask[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int64_t n = n0 + 64 * nh + 32 * j + (lane & 31);
    int b = 0, oh = 0, ow = 0;
    int64_t f0 = 0;
    const bool n_ok = n < a.N;
    if (n_ok) f0 = base_index(n, b, oh, ow);
    uint32_t m = 0;
#pragma unroll
    for (int t = 0; t < TAPS; ++t) {
      const int kh = t / KW, kw = t % KW;
      const int ih = oh - pad + kh, iw = ow - pad + kw;
      if (n_ok && ih >= 0 && ih < H && iw >= 0 && iw < W) m |= 1u << t;
    }
    vmask[j] = m;
    row_addr[j] = (int)(f0 - f_lo) * row_stride + lane_off;
  }

  RowMeta rm;
  if (wave_on) load_row_meta(a, mt, lane, rm);

  v16i acc[2];
  for (int j = 0; j < 2; ++j)
    for (int r = 0; r < 16; ++r) acc[j][r] = 0;

  __syncthreads();  // patch is in LDS

  if (wave_on) {
    if (kind == TILE_NIB_SHIFT)
      patch_mainloop<TILE_NIB_SHIFT, TAPS, CPT>(lane_ptr, T, smem, row_addr, vmask, zaddr, W * row_stride, row_stride, acc);
    else if (kind == TILE_NIB_LUT)
      patch_mainloop<TILE_NIB_LUT, TAPS, CPT>(lane_ptr, T, smem, row_addr, vmask, zaddr, W * row_stride, row_stride, acc);
    else
      patch_mainloop<TILE_I8, TAPS, CPT>(lane_ptr, T, smem, row_addr, vmask, zaddr, W * row_stride, row_stride, acc);
  }

  // ---- add the two partial sums of a pair: each wave hands over the block it does not finish
  __syncthreads();  // everyone is done with the patch; LDS is reused for the exchange
  {
    int* xch = (int*)smem + wave * (16 * LANES);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      v4i give;
#pragma unroll
      for (int e = 0; e < 4; ++e) give[e] = parity ? acc[0][4 * q + e] : acc[1][4 * q + e];
      *(v4i*)(xch + q * (4 * LANES) + lane * 4) = give;
    }
  }
  __syncthreads();
  if (!wave_on) return;
  {
    const int partner = wave ^ 4;
    const int* xch = (const int*)smem + partner * (16 * LANES);
    v16i mine;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const v4i got = *(const v4i*)(xch + q * (4 * LANES) + lane * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) mine[4 * q + e] = (parity ? acc[1][4 * q + e] : acc[0][4 * q + e]) + got[e];
    }
    finish_tile(a, kind, mine, rm, n0 + 64 * nh + 32 * parity + (lane & 31));
  }
}

// Geometry checks for the LDS-resident kernel; fills the LDS layout when it applies.
static bool patch_kernel_applies(const GemmArgs& a, int* row_stride, int* patch_rows, size_t* lds_bytes) {
  if (!a.conv || a.ep.act_bits != 4 || a.d.stride != 1) return false;
  const int taps = a.d.KH * a.d.KW;
  if (!(taps == 1 || (a.d.KH == 3 && a.d.KW == 3))) return false;
  if (a.d.C != 64 && a.d.C != 128 && a.d.C != 256 && a.d.C != 512) return false;
  // the flattened input index of a tile's pixels must grow with the pixel number
  if (a.OH > a.d.H || a.OW > a.d.W) return false;
  // widest run of flattened input pixels any 128-pixel tile touches
  const int64_t span = (int64_t)PT_BN + (int64_t)(a.d.KH - 1) * a.d.W + (a.d.KW - 1)
                       + (int64_t)(a.d.H - a.OH) * a.d.W * ((PT_BN + a.OH * a.OW - 1) / (a.OH * a.OW) + 1)
                       + (int64_t)(a.d.W - a.OW) * ((PT_BN + a.OW - 1) / a.OW + 1);
  const int rs = a.d.C + 16;
  const size_t need = (size_t)(span + 1) * rs;
  const size_t xch = 8 * 16 * LANES * 4;
  if (need > 150 * 1024) return false;
  *row_stride = rs;
  *patch_rows = (int)span;
  *lds_bytes = need > xch ? need : xch;
  return true;
}

// Dynamic LDS above 64 KiB must be allowed per kernel once (per device); remember what was set.
template <int TAPS, int CPT>
static int launch_patch_t(const GemmArgs& a, int row_stride, int patch_rows, size_t lds, dim3 grid, hipStream_t s) {
  static bool allowed[64] = {false};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= 64) return (int)hipErrorInvalidDevice;
  if (!allowed[dev]) {
    e = hipFuncSetAttribute((const void*)conv_patch_kernel<TAPS, CPT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024);
    if (e != hipSuccess) return (int)e;
    allowed[dev] = true;
  }
  hipLaunchKernelGGL((conv_patch_kernel<TAPS, CPT>), grid, dim3(512), lds, s, a, row_stride, patch_rows);
  return (int)hipGetLastError();
}

static int launch_patch(const GemmArgs& a, int row_stride, int patch_rows, size_t lds, hipStream_t s) {
  dim3 grid((unsigned)((a.N + PT_BN - 1) / PT_BN), (unsigned)((a.w.n_tiles + 1) / 2), 1);
  const int taps = a.d.KH * a.d.KW;
  const int cpt = a.d.C / KSTEP;
#define RMSMP_PATCH_CASE(TP, CP) \
  if (taps == TP && cpt == CP) return launch_patch_t<TP, CP>(a, row_stride, patch_rows, lds, grid, s);
  RMSMP_PATCH_CASE(9, 2)
  RMSMP_PATCH_CASE(9, 4)
  RMSMP_PATCH_CASE(9, 8)
  RMSMP_PATCH_CASE(9, 16)
  RMSMP_PATCH_CASE(1, 2)
  RMSMP_PATCH_CASE(1, 4)
  RMSMP_PATCH_CASE(1, 8)
  RMSMP_PATCH_CASE(1, 16)
#undef RMSMP_PATCH_CASE
  return (int)hipErrorInvalidValue;
}

int launch_gemm(const GemmArgs& a, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  if (a.N <= 0) return 0;
  if (a.conv) {
    int rs, pr;
    size_t lds;
    if (patch_kernel_applies(a, &rs, &pr, &lds)) return launch_patch(a, rs, pr, lds, s);
    return a.ep.act_bits == 4 ? launch_general<4, true, true>(a, s) : launch_general<8, true, true>(a, s);
  }
  const bool vec = (a.K % 16) == 0;
  if (a.ep.act_bits == 4) return vec ? launch_general<4, false, true>(a, s) : launch_general<4, false, false>(a, s);
  return vec ? launch_general<8, false, true>(a, s) : launch_general<8, false, false>(a, s);
}

// ---------------------------------------------------------------- explicit im2col
//
// Fallback for layers whose channel count is not a multiple of 16: writes the lowered matrix
// [N][Kpad] in the K order the weights are stored in, (kh, kw) outer and channel inner.
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
