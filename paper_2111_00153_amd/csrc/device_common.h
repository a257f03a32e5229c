// Device-side helpers shared by the kernels of librmsmp (gfx950): MFMA operand types, register-level
// decode of the three storage classes, tile lookup and the fused epilogue (zero point, per-row
// scale, bias, ReLU, 4-bit requantization).  Included by every .hip file that holds a GEMM kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>

#include "phase_stamps.h"
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
// same, from a wave-uniform base and a 32-bit per-lane byte offset
template <int KIND>
__device__ __forceinline__ typename RawFrag<KIND>::type load_raw(const uint8_t* uniform_base, uint32_t lane_off) {
  return *(const typename RawFrag<KIND>::type*)(uniform_base + lane_off);
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

// ---------------------------------------------------------------- tile lookup

// Class, live rows and blob offset of weight tile mt, from the class sizes alone (no memory access).
__device__ __forceinline__ TileRef tile_ref(const DevicePacked& w, int mt) {
  const int64_t nib_tile = (int64_t)w.nks * LANES * 8, i8_tile = (int64_t)w.nks * LANES * 16;
  const int t0 = w.class_tiles[0], t1 = w.class_tiles[1];
  TileRef t;
  int idx;
  if (mt < t0) {
    t.kind = TILE_NIB_SHIFT;
    idx = mt;
    t.blob_off = (int64_t)mt * nib_tile;
  } else if (mt < t0 + t1) {
    t.kind = TILE_NIB_LUT;
    idx = mt - t0;
    t.blob_off = (int64_t)mt * nib_tile;
  } else {
    t.kind = TILE_I8;
    idx = mt - t0 - t1;
    t.blob_off = (int64_t)(t0 + t1) * nib_tile + (int64_t)idx * i8_tile;
  }
  // (selected, not indexed: an index into the kernel arguments would be one more dependent read)
  const int rows0 = w.class_rows[0], rows1 = w.class_rows[1], rows2 = w.class_rows[2];
  const int left = (t.kind == TILE_NIB_SHIFT ? rows0 : t.kind == TILE_NIB_LUT ? rows1 : rows2) - idx * TILE_M;
  t.nvalid = left < TILE_M ? left : TILE_M;
  return t;
}

// ---------------------------------------------------------------- epilogue

// Every fp32 operation is rounded on its own so that codes are reproducible bit for bit.
// What the epilogue needs from the kernel arguments.  Kernel arguments are fetched with scalar
// loads where they are first used; at the end of a kernel that is a cold miss in front of the
// stores, so kernels copy these fields at their start and pin them in registers.
// The epilogue's pointers pass through an empty asm (see pin_epilogue_args), which hides from the
// compiler that they point to global memory; without the explicit address space it would emit
// flat loads and stores, whose completion it cannot count and therefore waits for in full.
#define RMSMP_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ RMSMP_GLOBAL T* as_global(T* p) {
  return (RMSMP_GLOBAL T*)p;
}
typedef unsigned v2u __attribute__((ext_vector_type(2)));

struct EpArgs {
  void* Y;
  const float* bias;
  int64_t N, M;
  float act_scale, out_inv_scale;
  int zp, relu, out_kind, out_zero_point;
};

__device__ __forceinline__ EpArgs pin_epilogue_args(const GemmArgs& a) {
  EpArgs e;
  e.Y = a.Y;
  e.bias = a.ep.bias;
  e.N = a.N;
  e.M = a.M;
  e.act_scale = a.ep.act_scale;
  e.out_inv_scale = a.ep.out_inv_scale;
  e.zp = a.ep.act_zero_point;
  e.relu = a.ep.relu;
  e.out_kind = a.ep.out_kind;
  e.out_zero_point = a.ep.out_zero_point;
  // an empty asm that "modifies" the values keeps the loads here
  asm volatile("" : "+s"(e.Y), "+s"(e.bias), "+s"(e.N), "+s"(e.M), "+s"(e.act_scale), "+s"(e.out_inv_scale), "+s"(e.zp),
               "+s"(e.relu), "+s"(e.out_kind), "+s"(e.out_zero_point));
  return e;
}

// Row metadata of the 16 consecutive grouped rows a lane finishes, held in registers:
// {rowscale bits, rowsum, original row (-1 = padding), grouped position} per row.
struct RowMeta {
  int4 m[16];
  __device__ __forceinline__ int scale_bits(int r) const { return m[r].x; }
  __device__ __forceinline__ int rowsum(int r) const { return m[r].y; }
  __device__ __forceinline__ int orig(int r) const { return m[r].z; }
  __device__ __forceinline__ int gpos0() const { return m[0].w; }
};

// The same, read on demand from a table in LDS laid out field by field (rows x 4 fields): an
// epilogue then only touches the fields its output kind needs and keeps few of them in registers.
struct RowMetaLds {
  const int* base;  // LDS: field f of the lane's row r at base[f * rows + r]
  int rows;
  __device__ __forceinline__ int scale_bits(int r) const { return base[r]; }
  __device__ __forceinline__ int rowsum(int r) const { return base[rows + r]; }
  __device__ __forceinline__ int orig(int r) const { return base[2 * rows + r]; }
  __device__ __forceinline__ int gpos0() const { return base[3 * rows]; }
};

__device__ __forceinline__ void load_row_meta(const DevicePacked& w, int mt, int lane, RowMeta& rm) {
  const int4* src = (const int4*)w.p_meta + (int64_t)mt * TILE_M + 16 * (lane >> 5);
#pragma unroll
  for (int r = 0; r < 16; ++r) rm.m[r] = src[r];
}

// 4-bit output codes of one pixel block: clamp(rint(y * inv_s), 0, 15) for the lane's 16 rows,
// row r in nibble r of the 64-bit result.  BIAS / RELU say which of the optional steps exist, so
// that the common cases carry no dead instructions.  The float-to-byte conversion packs a value
// itself: v_cvt_pk_u8_f32 rounds to nearest even and clamps to [0, 255].
template <bool BIAS, bool RELU>
__device__ __forceinline__ void requant_block(const v16i& v, const float (&m)[16], const float (&bias)[16], float inv_s,
                                              uint32_t (&packed)[2]) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    uint32_t even = 0u, odd = 0u;  // bytes: rows 8h + {0,2,4,6} and 8h + {1,3,5,7}
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = 8 * h + i;
      float y = __fmul_rn((float)v[r], m[r]);
      if (BIAS) y = __fadd_rn(y, bias[r]);
      if (RELU) y = fmaxf(y, 0.0f);
      // the conversion below rounds half to even and saturates at 0 (checked against rint + clamp
      // over a dense sweep of [0, 16) and every half-way case up to 300), so only the upper clamp
      // is left to do here
      const float t = fminf(__fmul_rn(y, inv_s), 15.0f);
      if (i & 1)
        odd = __builtin_amdgcn_cvt_pk_u8_f32(t, i >> 1, odd);
      else
        even = __builtin_amdgcn_cvt_pk_u8_f32(t, i >> 1, even);
    }
    packed[h] = even | (odd << 4);
  }
}

// GELU + affine 4-bit code of one pixel block (out_kind 3): g = y * Phi(y) in float64 rounded to
// fp32, code = clamp(rint(g * inv_s) + z, 0, 15).  As a function of the fp32 pre-activation y the
// code is piecewise constant, and the host has found its break points exactly (GeluTable, handed
// over inside the kernel arguments): for y at or above the minimum of GELU the code is the largest
// c with rise[c] <= y, searched downwards from the code y itself would get (never too low, since
// GELU(y) <= max(y, 0)); below the minimum it is fall_base plus the number of fall[j] >= y.
// KOFF: byte offset of the GemmArgs block inside the kernel arguments (0 unless the kernel takes
// leading scalar arguments in front of it).
template <int KOFF = 0>
__device__ __forceinline__ void gelu_requant_block(const v16i& v, const float (&m)[16], const float (&bias)[16], float inv_s,
                                                   int z_out, uint32_t (&packed)[2]) {
  // (the table is read in place: scalar loads for the wave-uniform fields, a per-lane load for rise[code])
  typedef const __attribute__((address_space(4))) char karg_char;
  typedef const __attribute__((address_space(4))) GeluTable karg_table;
  karg_table* const tab = (karg_table*)((karg_char*)__builtin_amdgcn_kernarg_segment_ptr() + KOFF + __builtin_offsetof(GemmArgs, gelu));
  const float y_split = tab->y_split;
  const int fix_steps = tab->fix_steps, fall_base = tab->fall_base, n_fall = tab->n_fall;
  const RMSMP_GLOBAL float* const rise = (const RMSMP_GLOBAL float*)(uintptr_t)tab->rise;
  // eight rows at a time (one output word): half the live registers of doing all sixteen at once
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    int code[8];
    float y[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = 8 * h + i;
      y[i] = __fadd_rn(__fmul_rn((float)v[r], m[r]), bias[r]);
      const float t = fminf(__fmul_rn(fmaxf(y[i], 0.0f), inv_s), 15.0f);
      const int c = (int)__builtin_rintf(t) + z_out;
      code[i] = c < 15 ? c : 15;
    }
#pragma unroll 1
    for (int s = 0; s < fix_steps; ++s) {
#pragma unroll
      for (int i = 0; i < 8; ++i) code[i] -= (y[i] < rise[code[i]]) ? 1 : 0;
    }
    if (n_fall > 0) {
      int cf[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) cf[i] = fall_base;
#pragma unroll 1
      for (int j = 0; j < n_fall; ++j) {
        const float f = tab->fall[j];
#pragma unroll
        for (int i = 0; i < 8; ++i) cf[i] += (y[i] <= f) ? 1 : 0;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) code[i] = y[i] < y_split ? cf[i] : code[i];
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) code[i] = y[i] < y_split ? fall_base : code[i];
    }
    uint32_t w = 0u;
#pragma unroll
    for (int i = 0; i < 8; ++i) w |= (uint32_t)code[i] << (4 * i);
    packed[h] = w;
  }
}

// Finish NB 32x32 accumulator tiles of the same weight tile (NB pixel blocks): zero-point
// correction, per-row scale, bias, ReLU, then int32 / fp32 / nibble-packed 4-bit store.
// Register r of lane l is grouped row 16*(l/32)+r of the weight tile and column n[j]; the 16
// registers of a lane are 16 consecutive grouped rows.  n_rows = how many of the lane's 16 rows
// exist (live rows of a tile are a prefix).  Straight-line code: padding rows are computed and
// dropped at the store, and all results are formed before the first store is issued (a store
// pins its data registers until it has left, so interleaving would stall on every block).
//
// Accumulators of shift-decoded tiles are 16 times the true sums.  The integer output divides
// them (an exact shift); the float paths fold the factor into the per-row multiplier instead:
// float(16 a) * (m / 16) and float(a) * m are the same float, because scaling by a power of two
// commutes with rounding.
// GELU: whether the calling kernel carries the GELU epilogue (out_kind 3) at all.
template <int NB, class Meta, bool GELU = true, int KOFF = 0>
__device__ __forceinline__ void finish_tiles(const EpArgs& a, int kind, const v16i (&acc)[NB], const Meta& rm,
                                             int n_rows, const int64_t (&n)[NB]) {
  if (n_rows <= 0) return;
  const int zp = a.zp;
  const bool has_bias = a.bias != nullptr;
  const bool relu = a.relu != 0;
  const int out_kind = a.out_kind;
  const bool x16 = kind == TILE_NIB_SHIFT;
  v16i v[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) v[j] = acc[j];
  if (out_kind == 0) {
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int s = (x16 ? v[j][r] >> 4 : v[j][r]) - zp * rm.rowsum(r);
        if (r < n_rows && n[j] < a.N) as_global((int32_t*)a.Y)[(int64_t)rm.orig(r) * a.N + n[j]] = s;
      }
    return;
  }
  if (zp != 0) {
    const int zs = x16 ? 16 * zp : zp;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int c = zs * rm.rowsum(r);
#pragma unroll
      for (int j = 0; j < NB; ++j) v[j][r] -= c;
    }
  }
  float bias[16], m[16];
  const float fold = x16 ? 0.0625f : 1.0f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    bias[r] = 0.0f;
    m[r] = __fmul_rn(__fmul_rn(__int_as_float(rm.scale_bits(r)), a.act_scale), fold);
  }
  if (has_bias) {
#pragma unroll
    for (int r = 0; r < 16; ++r) bias[r] = as_global(a.bias)[rm.orig(r) < 0 ? 0 : rm.orig(r)];
  }
  if (out_kind == 1) {
    // adding a zero bias and taking the maximum with -inf change nothing, so one code path serves
    // every combination of the two options
    const float floor_y = relu ? 0.0f : -__builtin_inff();
    float y[NB][16];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) y[j][r] = fmaxf(__fadd_rn(__fmul_rn((float)v[j][r], m[r]), bias[r]), floor_y);
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (r < n_rows && n[j] < a.N) as_global((float*)a.Y)[(int64_t)rm.orig(r) * a.N + n[j]] = y[j][r];
    return;
  }
  // with a positive output scale the clamp at code 0 already does what ReLU would (a negative y
  // rounds to a non-positive value), so the separate maximum is skipped
  const bool relu_q = relu && !(a.out_inv_scale > 0.0f);
  uint32_t packed[NB][2];
  if (GELU && out_kind == 3) {
#pragma unroll
    for (int j = 0; j < NB; ++j) gelu_requant_block<KOFF>(v[j], m, bias, a.out_inv_scale, a.out_zero_point, packed[j]);
  } else {
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    if (has_bias) {
      if (relu_q)
        requant_block<true, true>(v[j], m, bias, a.out_inv_scale, packed[j]);
      else
        requant_block<true, false>(v[j], m, bias, a.out_inv_scale, packed[j]);
    } else {
      if (relu_q)
        requant_block<false, true>(v[j], m, bias, a.out_inv_scale, packed[j]);
      else
        requant_block<false, false>(v[j], m, bias, a.out_inv_scale, packed[j]);
    }
  }
  }
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    if (n[j] >= a.N) continue;
    // the first grouped position of a lane is a multiple of 16
    RMSMP_GLOBAL uint8_t* dst = as_global((uint8_t*)a.Y) + n[j] * (a.M / 2) + (rm.gpos0() >> 1);
    if (n_rows == 16 && (((uintptr_t)dst) & 7) == 0) {
      *(RMSMP_GLOBAL v2u*)dst = (v2u){packed[j][0], packed[j][1]};
    } else {
      for (int b = 0; b < n_rows / 2; ++b) dst[b] = (uint8_t)(packed[j][b >> 2] >> (8 * (b & 3)));
    }
  }
}

__device__ __forceinline__ int lane_rows(int nvalid, int lane) {
  const int left = nvalid - 16 * (lane >> 5);
  return left < 0 ? 0 : left > 16 ? 16 : left;
}

}  // namespace rmsmp
