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
#include <type_traits>

#include "rmsmp_internal.h"

namespace rmsmp {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Optional per-wave phase timestamps for tuning builds (-DRMSMP_PHASE_TIMING); compiled out
// otherwise.  A stamp is one clock read parked in the first KiB of dynamic LDS (16 slots per
// wave); the kernel copies the slots to g_phase_buf when it ends, so a stamp costs no memory
// round trip where it is taken.
#ifdef RMSMP_PHASE_TIMING
__device__ unsigned long long* g_phase_buf = nullptr;
constexpr int PHASE_LDS_BYTES = 1024;
extern __shared__ __attribute__((aligned(16))) uint8_t phase_smem[];
#define RMSMP_PHASE(id)                                                                                  \
  do {                                                                                                   \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
    if ((threadIdx.x & 63) == 0) ((unsigned long long*)phase_smem)[(threadIdx.x >> 6) * 16 + (id)] = clock64(); \
    __builtin_amdgcn_sched_barrier(0);                                                                   \
  } while (0)
#define RMSMP_PHASE_FLUSH()                                                                              \
  do {                                                                                                   \
    if (g_phase_buf && (threadIdx.x & 63) == 0)                                                          \
      for (int i_ = 0; i_ < 16; ++i_)                                                                    \
        g_phase_buf[(blockIdx.x * 8 + (threadIdx.x >> 6)) * 16 + i_] =                                  \
            ((unsigned long long*)phase_smem)[(threadIdx.x >> 6) * 16 + i_];                             \
  } while (0)
#else
constexpr int PHASE_LDS_BYTES = 0;
#define RMSMP_PHASE(id) \
  do {                  \
  } while (0)
#define RMSMP_PHASE_FLUSH() \
  do {                      \
  } while (0)
#endif

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
  const int left = w.class_rows[t.kind] - idx * TILE_M;
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
  int zp, relu, out_kind;
  bool stamps = false;  // tuning builds: this kernel reserved the stamp slots in LDS
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
  // an empty asm that "modifies" the values keeps the loads here
  asm volatile("" : "+s"(e.Y), "+s"(e.bias), "+s"(e.N), "+s"(e.M), "+s"(e.act_scale), "+s"(e.out_inv_scale), "+s"(e.zp),
               "+s"(e.relu), "+s"(e.out_kind));
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
// that is already an exact integer in [0, 15], so its own rounding mode plays no role.
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
      const float t = __builtin_amdgcn_fmed3f(rintf(__fmul_rn(y, inv_s)), 0.0f, 15.0f);
      if (i & 1)
        odd = __builtin_amdgcn_cvt_pk_u8_f32(t, i >> 1, odd);
      else
        even = __builtin_amdgcn_cvt_pk_u8_f32(t, i >> 1, even);
    }
    packed[h] = even | (odd << 4);
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
template <int NB, class Meta>
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
  if (a.stamps) RMSMP_PHASE(8);
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
  if (a.stamps) RMSMP_PHASE(12);
  // with a positive output scale the clamp at code 0 already does what ReLU would (a negative y
  // rounds to a non-positive value), so the separate maximum is skipped
  const bool relu_q = relu && !(a.out_inv_scale > 0.0f);
  uint32_t packed[NB][2];
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
  if (a.stamps) RMSMP_PHASE(13);
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
  if (a.stamps) RMSMP_PHASE(9);
}

__device__ __forceinline__ int lane_rows(int nvalid, int lane) {
  const int left = nvalid - 16 * (lane >> 5);
  return left < 0 ? 0 : left > 16 ? 16 : left;
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
__device__ __forceinline__ void general_slab_mfma(uint4 T, const uint8_t* sB, int lane, v16i (&acc)[2],
                                                  typename RawFrag<KIND>::type w0, typename RawFrag<KIND>::type w1) {
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
  const EpArgs ea = pin_epilogue_args(a);

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
  const TileRef tr = tile_ref(a.w, wave_on ? mt : 0);
  const int kind = tr.kind;
  uint4 T = make_uint4(0, 0, 0, 0);
  if (wave_on && kind == TILE_NIB_LUT)
    T = *(const uint4*)(a.w.p_lut + ((int64_t)mt * TILE_M + tile_row_goff(lane & 31)) * 4);
  const int frag_bytes = kind == TILE_I8 ? 16 : 8;
  const uint8_t* lane_ptr = a.w.blob + tr.blob_off + (int64_t)lane * frag_bytes;
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
        general_slab_mfma<TILE_NIB_SHIFT>(T, sB, lane, acc, make_uint2(raw0.x, raw0.y), make_uint2(raw1.x, raw1.y));
      else if (kind == TILE_NIB_LUT)
        general_slab_mfma<TILE_NIB_LUT>(T, sB, lane, acc, make_uint2(raw0.x, raw0.y), make_uint2(raw1.x, raw1.y));
      else
        general_slab_mfma<TILE_I8>(T, sB, lane, acc, raw0, raw1);
    }
  }

  if (!wave_on) return;
  RowMeta rm;
  load_row_meta(a.w, mt, lane, rm);
  const int n_rows = lane_rows(tr.nvalid, lane);
  const int64_t ncol[2] = {n0 + (lane & 31), n0 + 32 + (lane & 31)};
  finish_tiles<2>(ea, kind, acc, rm, n_rows, ncol);
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
// shared by both weight tiles whatever their class.
//
// Four waves, one per SIMD.  A wave owns a 64-row x 64-pixel block (two weight fragments from
// registers, two activation fragments from LDS, four MFMAs per K step, so each LDS byte and
// each weight byte feeds two MFMAs) and every other K step; the two partial sums of a block are
// added through LDS at the end (int32 addition is exact in any order).  The decode and address
// arithmetic of a step are independent of its MFMAs and issue in their shadow.
//
// The two tiles of a work-group are tile y and tile (n_tiles-1-y): tiles are sorted by class,
// so a table-decoded (PoT) tile, whose decode is the most expensive, is paired with a cheap one
// whenever the layer has both, and no work-group is left with two expensive tiles.
//
// Packed weights stream from global memory straight into a register ring that runs PT_RING
// steps ahead of the MFMAs.  A kernel starts with cold caches, so every global read that does
// not depend on another is issued up front (ring, row metadata, the whole patch): one memory
// latency is paid.  The K loop is fully unrolled straight-line code: with branches in it the
// compiler can no longer count outstanding loads and waits for all of them at every step, and a
// rolled loop makes it copy the ring registers at the back edge, which drains the ring as well.
constexpr int PT_THREADS = 256;
// K split KS: how many waves share one 64x64 output block, each taking every KS-th K step.
// KS = 2: work-group = 128 pixels (two blocks side by side); KS = 4: 64 pixels, for grids too
// small to put two work-groups on a compute unit otherwise (a wave issues in order and cannot
// hide its own decode behind its own MFMAs; a second wave on the SIMD can).
constexpr int pt_bn(int ks) { return 64 * (4 / ks); }
// bytes of the partial-sum exchange buffer: every wave parks the quarters of its block it does not finish
constexpr int pt_xch_bytes(int ks) { return 4 * (4 - 4 / ks) * 16 * LANES * 4; }
constexpr int PT_PATCH_UNROLL = 6;              // 16-byte patch pieces in flight per thread
constexpr int PT_META_BYTES = 2 * TILE_M * 16;  // row metadata of the work-group's 64 rows, kept at the start of LDS
#ifndef RMSMP_PT_RING
#define RMSMP_PT_RING 4
#endif
constexpr int PT_RING = RMSMP_PT_RING;          // K steps of packed weights in flight per wave and tile

struct PatchGeom {
  int gx, gy;         // pixel tiles, work-groups per pixel tile (the launch grid is one-dimensional)
  int row_stride;     // LDS bytes per patch pixel (C + 16)
  int patch_rows;     // pixels staged per work-group
  uint32_t magic_hw;  // ceil(2^32 / (OH*OW)), 0 when OH*OW == 1
  uint32_t magic_ow;  // ceil(2^32 / OW), 0 when OW == 1
};

// n / d for n*d < 2^32 with magic = ceil(2^32/d) (0 stands for d == 1): one multiply.
__device__ __forceinline__ int fast_div(int n, uint32_t magic) {
  return magic ? (int)__umulhi((uint32_t)n, magic) : n;
}

// What the prologue leaves for the per-tile-pair part of the kernel.
struct PatchState {
  uint8_t* meta;   // LDS: row metadata of the current tile pair (64 rows x 16 bytes)
  uint8_t* xch;    // LDS: partial-sum exchange buffer (4 waves x 2 blocks x 4 KiB)
  uint8_t* patch;  // LDS: decoded input patch, then the zero-point row
  int row_addr0, row_addr1;  // per 32-pixel block of this lane
  uint32_t vmask0, vmask1;
  int zaddr;
  int n0;
};

// Everything a tile pair reads from global memory before its K loop, as raw registers: the
// first PT_RING K steps of both weight tiles of this wave, the lookup tables of table-decoded
// tiles and (threads 0..63) one row of metadata.  Issued as early as possible -- for the first
// pair together with the patch, for later pairs before the previous pair's epilogue -- so that
// the memory latency is hidden behind other work.  The tile classes are only known at run time
// here; 4-bit fragments use the first half of a slot.
struct PairLoads {
  uint4 ring0[PT_RING], ring1[PT_RING];
  uint4 T0, T1;
  int4 meta_row;
};

template <int NSTEP, int KS>
__device__ __forceinline__ void issue_ring(const uint8_t* wb, int kind, int lane, uint4 (&ring)[PT_RING]) {
  if (kind == TILE_I8) {
#pragma unroll
    for (int u = 0; u < PT_RING; ++u)
      if (u < NSTEP) ring[u] = *(const uint4*)(wb + (int64_t)u * KS * (LANES * 16) + (uint32_t)lane * 16);
  } else {
#pragma unroll
    for (int u = 0; u < PT_RING; ++u)
      if (u < NSTEP) {
        const uint2 w = *(const uint2*)(wb + (int64_t)u * KS * (LANES * 8) + (uint32_t)lane * 8);
        ring[u].x = w.x;
        ring[u].y = w.y;
      }
  }
}

template <int NSTEP, int KS>
__device__ __forceinline__ void issue_pair_loads(const GemmArgs& a, int mt0, int mt1, const TileRef& tr0, const TileRef& tr1,
                                                 PairLoads& pl) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int kq = __builtin_amdgcn_readfirstlane(tid >> 6) / (4 / KS);
  issue_ring<NSTEP, KS>(a.w.blob + tr0.blob_off + kq * (LANES * (tr0.kind == TILE_I8 ? 16 : 8)), tr0.kind, lane, pl.ring0);
  issue_ring<NSTEP, KS>(a.w.blob + tr1.blob_off + kq * (LANES * (tr1.kind == TILE_I8 ? 16 : 8)), tr1.kind, lane, pl.ring1);
  if (tr0.kind == TILE_NIB_LUT) pl.T0 = *(const uint4*)(a.w.p_lut + ((int64_t)mt0 * TILE_M + tile_row_goff(lane & 31)) * 4);
  if (tr1.kind == TILE_NIB_LUT) pl.T1 = *(const uint4*)(a.w.p_lut + ((int64_t)mt1 * TILE_M + tile_row_goff(lane & 31)) * 4);
  // threads 0..31 fetch tile 0's rows, 32..63 tile 1's
  if (tid < 2 * TILE_M)
    pl.meta_row = ((const int4*)a.w.p_meta)[(tid < TILE_M ? mt0 : mt1) * TILE_M + (tid & (TILE_M - 1))];
}

template <int KIND>
__device__ __forceinline__ typename RawFrag<KIND>::type raw_of(const uint4& r);
template <>
__device__ __forceinline__ uint2 raw_of<TILE_NIB_SHIFT>(const uint4& r) { return make_uint2(r.x, r.y); }
template <>
__device__ __forceinline__ uint2 raw_of<TILE_NIB_LUT>(const uint4& r) { return make_uint2(r.x, r.y); }
template <>
__device__ __forceinline__ uint4 raw_of<TILE_I8>(const uint4& r) { return r; }
__device__ __forceinline__ void raw_into(uint4& r, uint2 w) { r.x = w.x; r.y = w.y; }
__device__ __forceinline__ void raw_into(uint4& r, uint4 w) { r = w; }

// Which pair comes after the current one in this work-group (valid == false: none).
struct NextPair {
  bool valid;
  int mt0, mt1;
  TileRef tr0, tr1;
};

// What follows a tile pair's K loop: add the partial sums of the waves that share an output block,
// then the epilogue.  acc: [weight tile][pixel block] of this wave's 64x64 block.
template <int KS, bool MULTI, int KIND0, int KIND1>
__device__ __forceinline__ void pair_tail(const EpArgs& ea, const PatchState& ps, v16i (&acc)[2][2], const TileRef& tr0,
                                          const TileRef& tr1, bool two) {
  constexpr int NWT = 4 / KS;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wt = wave % NWT;
  const int kq = wave / NWT;
  // ---- add the KS partial sums of a block.  The block's four quarters (weight tile t, pixel
  // block j: quarter 2t + j) are shared out among the KS waves: wave kq finishes quarters
  // kq*OWN .. kq*OWN+OWN-1 and parks the others in LDS for their owners.  The roles are KS copies
  // of the code under a wave-uniform branch, so that which accumulators are given and which are
  // kept is static (selecting them per element would cost 64 instructions).
  constexpr int OWN = 4 / KS;  // quarters a wave finishes: 2 (one tile, both pixel blocks) or 1
  if (!MULTI) __syncthreads();  // the exchange buffer overlays the patch: every wave is done reading it
  v16i mine[OWN];
  auto exchange = [&](auto kq_tag) {
    constexpr int KQ = decltype(kq_tag)::value;
    // slot [wave of the block][given quarter, in increasing order], 16 registers x 64 lanes each
    int* const blk = (int*)ps.xch + wt * (KS * (4 - OWN) * 16 * LANES);
    {
      int* dst = blk + KQ * ((4 - OWN) * 16 * LANES);
      int gi = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (q / OWN == KQ) continue;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          v4i gq;
#pragma unroll
          for (int e = 0; e < 4; ++e) gq[e] = acc[q >> 1][q & 1][4 * c + e];
          *(v4i*)(dst + gi * (16 * LANES) + c * (4 * LANES) + lane * 4) = gq;
        }
        ++gi;
      }
    }
    __syncthreads();
    RMSMP_PHASE(4);
#pragma unroll
    for (int o = 0; o < OWN; ++o) {
      constexpr int q0 = KQ * OWN;
      const int q = q0 + o;
      mine[o] = acc[q >> 1][q & 1];
#pragma unroll
      for (int gk = 0; gk < KS; ++gk) {
        if (gk == KQ) continue;
        // where giver gk put quarter q: its given quarters are all but its own, in order
        const int gi = q < gk * OWN ? q : q - OWN;
        const int* src = blk + gk * ((4 - OWN) * 16 * LANES) + gi * (16 * LANES);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const v4i got = *(const v4i*)(src + c * (4 * LANES) + lane * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) mine[o][4 * c + e] += got[e];
        }
      }
    }
  };
  if (kq == 0)
    exchange(std::integral_constant<int, 0>{});
  else if (kq == 1)
    exchange(std::integral_constant<int, 1>{});
  else if (KS == 4 && kq == 2)
    exchange(std::integral_constant<int, KS == 4 ? 2 : 0>{});
  else if (KS == 4)
    exchange(std::integral_constant<int, KS == 4 ? 3 : 0>{});
  // the quarters this wave finishes belong to one weight tile
  const int my_tile = kq * OWN / 2;
  if (!(my_tile == 1 && !two)) {
    RMSMP_PHASE(5);
    RowMetaLds rm;
    rm.base = (const int*)__builtin_assume_aligned((const int*)ps.meta + my_tile * TILE_M + 16 * (lane >> 5), 64);
    rm.rows = 2 * TILE_M;
    const int n_rows = lane_rows(my_tile ? tr1.nvalid : tr0.nvalid, lane);
    const int kind = my_tile ? KIND1 : KIND0;
    const int64_t col0 = (int64_t)ps.n0 + 64 * wt + (lane & 31);
    if constexpr (OWN == 2) {
      const int64_t ncol[2] = {col0, col0 + 32};
      finish_tiles<2>(ea, kind, mine, rm, n_rows, ncol);
    } else {
      const int64_t ncol[1] = {col0 + 32 * (kq & 1)};
      finish_tiles<1>(ea, kind, mine, rm, n_rows, ncol);
    }
  }
}

// One tile pair: weight rings, K loop, partial-sum exchange, epilogue.  KIND0 / KIND1 are the
// storage classes of the two weight tiles (template parameters so that the K loop has no
// branches).
template <int TAPS, int CPT, int KIND0, int KIND1, bool MULTI, int KS>
__device__ __forceinline__ void patch_pair(const GemmArgs& a, const EpArgs& ea, const PatchGeom& g, const PatchState& ps,
                                           PairLoads& pl, const TileRef& tr0, const TileRef& tr1, bool two,
                                           const NextPair& next) {
  constexpr int KW = TAPS == 9 ? 3 : 1;
  constexpr int NKS = TAPS * CPT;
  constexpr int NSTEP = NKS / KS;  // K steps per wave
  constexpr int SPT = CPT / KS;    // of which per tap
  static_assert(CPT % KS == 0, "a tap must hold a whole number of K steps per wave");
  constexpr int NWT = 4 / KS;      // 64-pixel blocks side by side in the work-group
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wt = wave % NWT;  // which 64-pixel block of the work-group
  const int kq = wave / NWT;  // K steps kq, kq+KS, ...
  const int W = a.d.W;
  const int row_stride = g.row_stride;
  const uint8_t* smem = ps.patch;

  // ---- the weight rings were filled by issue_pair_loads; this wave's K steps continue from there
  constexpr int fb0 = KIND0 == TILE_I8 ? 16 : 8, fb1 = KIND1 == TILE_I8 ? 16 : 8;
  constexpr int step0 = LANES * fb0, step1 = LANES * fb1;  // bytes per K step
  // uniform base of this wave's first K step + 32-bit lane offset; stepping through K is scalar work
  const uint8_t* const wb0 = a.w.blob + tr0.blob_off + kq * step0;
  const uint8_t* const wb1 = a.w.blob + tr1.blob_off + kq * step1;
  const uint32_t wl0 = (uint32_t)lane * fb0, wl1 = (uint32_t)lane * fb1;
  const uint4 T0 = pl.T0, T1 = pl.T1;

  // LDS address of this lane's B fragment of pixel block j at tap t.  The tap of a step is known
  // at compile time (the same for both waves of a block); steps inside a tap differ by an
  // immediate offset and the per-wave part kq*KSTEP sits in the lane offsets.
  const int tap_row_bytes = W * row_stride;
  auto tap_base = [&](int t, int j) -> int {
    const int kh = t / KW, kw = t - kh * KW;
    const uint32_t vm = j ? ps.vmask1 : ps.vmask0;
    const int ra = j ? ps.row_addr1 : ps.row_addr0;
    return ((vm >> t) & 1u) ? ra + kh * tap_row_bytes + kw * row_stride : ps.zaddr;
  };

  RMSMP_PHASE(2);
  // ---- main loop over this wave's K steps; B fragments are fetched one step ahead
  v16i acc[2][2];  // [weight tile][pixel block]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
  {
    int cur0 = tap_base(0, 0), cur1 = tap_base(0, 1);
    v4i b0 = *(const v4i*)(smem + cur0);
    v4i b1 = *(const v4i*)(smem + cur1);
    // Software pipeline: step i multiplies with fragments decoded during step i-1 and decodes
    // those of step i+1, so the decode has no MFMA waiting for it.  A wave issues in order and
    // the matrix pipe takes one MFMA every 32 cycles, so four MFMAs in a row would block the
    // wave for 96 cycles; the scheduling groups below ask for the step's vector instructions to
    // be spread between its MFMAs instead, where they issue for free.
    v4i av0 = decode_raw<KIND0>(raw_of<KIND0>(pl.ring0[0]), T0);
    v4i av1 = decode_raw<KIND1>(raw_of<KIND1>(pl.ring1[0]), T1);
    if (PT_RING < NSTEP) {
      raw_into(pl.ring0[0], load_raw<KIND0>(wb0 + (int64_t)PT_RING * KS * step0, wl0));
      raw_into(pl.ring1[0], load_raw<KIND1>(wb1 + (int64_t)PT_RING * KS * step1, wl1));
    }
    constexpr int NV0 = KIND0 == TILE_NIB_SHIFT ? 6 : KIND0 == TILE_NIB_LUT ? 22 : 0;
    constexpr int NV1 = KIND1 == TILE_NIB_SHIFT ? 6 : KIND1 == TILE_NIB_LUT ? 22 : 0;
    constexpr int NVQ = (NV0 + NV1 + 4 + 3) / 4;  // vector instructions per MFMA slot
    // step i of this wave (K step 2*i + kq); everything indexed by i is static after unrolling
    auto step = [&](int i) {
      v4i nav0 = av0, nav1 = av1, nb0 = b0, nb1 = b1;
      if (i + 1 < NSTEP) {
        const int u = (i + 1) % PT_RING;
        nav0 = decode_raw<KIND0>(raw_of<KIND0>(pl.ring0[u]), T0);
        nav1 = decode_raw<KIND1>(raw_of<KIND1>(pl.ring1[u]), T1);
        if (i + 1 + PT_RING < NSTEP) {
          raw_into(pl.ring0[u], load_raw<KIND0>(wb0 + (int64_t)(i + 1 + PT_RING) * KS * step0, wl0));
          raw_into(pl.ring1[u], load_raw<KIND1>(wb1 + (int64_t)(i + 1 + PT_RING) * KS * step1, wl1));
        }
        if ((i + 1) % SPT == 0) {
          cur0 = tap_base((i + 1) / SPT, 0);
          cur1 = tap_base((i + 1) / SPT, 1);
        }
        nb0 = *(const v4i*)(smem + cur0 + ((i + 1) % SPT) * KS * KSTEP);
        nb1 = *(const v4i*)(smem + cur1 + ((i + 1) % SPT) * KS * KSTEP);
      }
      acc[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av1, b1, acc[1][1], 0, 0, 0);
      av0 = nav0;
      av1 = nav1;
      b0 = nb0;
      b1 = nb1;
      // desired issue order of this step: MFMA, a quarter of the vector work, MFMA, ...
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);    // the two LDS reads of the next B fragments
      __builtin_amdgcn_sched_group_barrier(0x002, NVQ, 0);  // VALU
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, NVQ, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);    // the two ring loads
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, NVQ, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, NVQ, 0);
      // and nothing crosses into the next step: without this the scheduler also sinks the ring
      // loads next to their use and the ring degenerates to one or two loads in flight
      __builtin_amdgcn_sched_barrier(0);
    };
#pragma unroll
    for (int i = 0; i < NSTEP; ++i) step(i);
  }

  RMSMP_PHASE(3);
  // ---- the rings are drained: start the next pair's reads now, behind the exchange and epilogue
  if (MULTI && next.valid) issue_pair_loads<NSTEP, KS>(a, next.mt0, next.mt1, next.tr0, next.tr1, pl);
  pair_tail<KS, MULTI, KIND0, KIND1>(ea, ps, acc, tr0, tr1, two);
  RMSMP_PHASE(6);
}

// Everything a work-group does once, whatever its tile pairs: stage the input patch in LDS,
// work out each lane's LDS addresses, and (behind the first batch of patch reads) start the
// reads of the first tile pair.
template <int TAPS, int CPT, bool MULTI, int KS>
__device__ __forceinline__ void patch_prologue(const GemmArgs& a, const PatchGeom& g, PatchState& ps, PairLoads& pl,
                                               int first_mt0, int first_mt1, const TileRef& first_tr0,
                                               const TileRef& first_tr1) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
  constexpr int C = CPT * KSTEP;
  constexpr int KW = TAPS == 9 ? 3 : 1;
  constexpr int KH = KW;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wt = wave % (4 / KS);
  const int kq = wave / (4 / KS);
  const int H = a.d.H, W = a.d.W, pad = a.d.pad, S = a.d.stride;
  const int hw_out = a.OH * a.OW;
  const int row_stride = g.row_stride, patch_rows = g.patch_rows;
  ps.meta = smem_raw + PHASE_LDS_BYTES;
  // a work-group with one tile pair is done with the patch when it exchanges partial sums, so
  // the exchange buffer lies over it; with several pairs the patch has to survive
  ps.xch = ps.meta + PT_META_BYTES;
  ps.patch = MULTI ? ps.xch + pt_xch_bytes(KS) : ps.xch;
  uint8_t* const smem = ps.patch;

  // flattened input index of tap (0,0) for output pixel n (may be negative / out of image)
  auto base_index = [&](int n, int& oh, int& ow) -> int {
    const int b = fast_div(n, g.magic_hw);
    const int rem = n - b * hw_out;
    oh = fast_div(rem, g.magic_ow);
    ow = rem - oh * a.OW;
    return (b * H + (oh * S - pad)) * W + (ow * S - pad);
  };
  int toh, tow;
  int f_lo = base_index(ps.n0, toh, tow);
  if (f_lo < 0) f_lo = 0;

  constexpr int NSTEP = TAPS * CPT / KS;

  // ---- 1. the patch.  Pixels f_lo .. f_lo+patch_rows-1 are one contiguous byte range of X;
  // piece idx (32 channels, 16 bytes) sits at byte 16*idx of it and goes, decoded to int8, to LDS
  // byte 32*idx + 16*(idx / pieces-per-pixel) (rows are padded by 16 bytes).  Reads past the end
  // of X are clamped (those rows are never used).  The first batch of loads is issued before
  // anything else in the kernel.
  {
    const uint8_t* X = (const uint8_t*)a.X;
    constexpr int PIECES = C / 32;
    const int total = patch_rows * PIECES;
    const int64_t x_bytes = (int64_t)a.d.B * H * W * (C / 2);
    const int64_t src0 = (int64_t)f_lo * (C / 2);
    auto put_piece = [&](int idx, uint4 w) {
      uint8_t* dst = smem + idx * 32 + (idx / PIECES) * 16;
      *(v4i*)dst = decode_act_u4(make_uint2(w.x, w.y));
      *(v4i*)(dst + 16) = decode_act_u4(make_uint2(w.z, w.w));
    };
    RMSMP_PHASE(15);
#pragma unroll 1
    for (int base = 0; base < total; base += PT_THREADS * PT_PATCH_UNROLL) {
      uint4 pw[PT_PATCH_UNROLL];
#pragma unroll
      for (int u = 0; u < PT_PATCH_UNROLL; ++u) {
        int64_t off = src0 + (int64_t)(base + u * PT_THREADS + tid) * 16;
        off = off < x_bytes - 16 ? off : x_bytes - 16;
        pw[u] = *(const uint4*)(X + off);
      }
      // behind the first batch of patch reads: everything the first tile pair needs
      if (base == 0) issue_pair_loads<NSTEP, KS>(a, first_mt0, first_mt1, first_tr0, first_tr1, pl);
      RMSMP_PHASE(7);
#pragma unroll
      for (int u = 0; u < PT_PATCH_UNROLL; ++u) {
        const int idx = base + u * PT_THREADS + tid;
        if (idx < total) put_piece(idx, pw[u]);
      }
    }
    // a constant row behind the patch: the zero-point code, for out-of-image taps
    const uint32_t zf = 0x01010101u * (uint32_t)(a.ep.act_zero_point & 15);
    if (tid < C / 16) *(v4i*)(smem + patch_rows * row_stride + tid * 16) = (v4i){(int)zf, (int)zf, (int)zf, (int)zf};
  }
  RMSMP_PHASE(11);

  // ---- 2. per lane and 32-pixel block: LDS address of tap (0,0) and the taps inside the image.
  // Validity is separable: tap (kh,kw) is inside iff kh is in [kh_lo,kh_hi] and kw in [kw_lo,kw_hi].
  const int lane_off = 16 * (lane >> 5) + kq * KSTEP;
  ps.zaddr = patch_rows * row_stride + lane_off;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = ps.n0 + 64 * wt + 32 * j + (lane & 31);
    const bool n_ok = n < (int)a.N;
    int oh = 0, ow = 0;
    const int f0 = base_index(n_ok ? n : ps.n0, oh, ow);
    const int kw_lo = max(0, pad - ow * S), kw_hi = min(KW - 1, W - 1 + pad - ow * S);
    const int kh_lo = max(0, pad - oh * S), kh_hi = min(KH - 1, H - 1 + pad - oh * S);
    const uint32_t wbits = kw_hi >= kw_lo ? ((2u << kw_hi) - (1u << kw_lo)) : 0u;  // bits kw_lo..kw_hi
    uint32_t m = 0;
#pragma unroll
    for (int kh = 0; kh < KH; ++kh) m |= (kh >= kh_lo && kh <= kh_hi) ? wbits << (KW * kh) : 0u;
    (j ? ps.vmask1 : ps.vmask0) = n_ok ? m : 0u;
    (j ? ps.row_addr1 : ps.row_addr0) = (f0 - f_lo) * row_stride + lane_off;
  }
  RMSMP_PHASE(1);

}

// The part of a work-group's life spent on tile pairs of one class combination: the prologue if
// this is where the work-group starts, then pair after pair while the classes stay the same.
// Returns the first pair not done.  A work-group normally stays inside one instance of this
// function from start to end, so that its instruction stream is one contiguous run of code: a
// kernel starts with cold instruction caches too, and every jump to code not yet fetched costs
// a memory round trip.
template <int TAPS, int CPT, int KIND0, int KIND1, bool MULTI, int KS>
__device__ __forceinline__ int patch_body(const GemmArgs& a, const EpArgs& ea, const PatchGeom& g, PatchState& ps,
                                          PairLoads& pl, bool first, int pi, int pair_hi) {
  const int tid = threadIdx.x;
  int mt0 = pi, mt1 = a.w.n_tiles - 1 - pi;
  TileRef tr0 = tile_ref(a.w, mt0), tr1 = tile_ref(a.w, mt1);
  if (first) patch_prologue<TAPS, CPT, MULTI, KS>(a, g, ps, pl, mt0, mt1, tr0, tr1);
#pragma unroll 1
  for (;;) {
    NextPair next;
    next.valid = MULTI && pi + 1 < pair_hi;
    next.mt0 = next.valid ? pi + 1 : mt0;
    next.mt1 = a.w.n_tiles - 1 - next.mt0;
    next.tr0 = tile_ref(a.w, next.mt0);
    next.tr1 = tile_ref(a.w, next.mt1);
    const bool two = mt1 > mt0;
    // everyone is done with the previous pair's metadata and exchange buffer, and (first pair)
    // the patch is complete
    __syncthreads();
    // row metadata parked in LDS until the epilogue (read after the exchange barrier)
    if (tid < 2 * TILE_M) {
      int* mf = (int*)ps.meta + tid;  // field by field: [field][64 rows]
      mf[0] = pl.meta_row.x;
      mf[2 * TILE_M] = pl.meta_row.y;
      mf[4 * TILE_M] = pl.meta_row.z;
      mf[6 * TILE_M] = pl.meta_row.w;
    }
    patch_pair<TAPS, CPT, KIND0, KIND1, MULTI, KS>(a, ea, g, ps, pl, tr0, tr1, two, next);
    ++pi;
    if (!next.valid) break;
    mt0 = next.mt0;
    mt1 = next.mt1;
    tr0 = next.tr0;
    tr1 = next.tr1;
    if (tr0.kind != KIND0 || tr1.kind != KIND1) break;
  }
  return pi;
}

// pairs_per_wg: how many tile pairs a work-group runs through against the same patch (large M).
// Pair y is tile y and tile n_tiles-1-y; the middle tile of an odd count stands alone (its second
// tile shadows it and is never stored).  Tiles are sorted by class, so kind0 <= kind1.
// MULTI = false is the one-pair-per-work-group build: no pair loop and no prefetch of a next
// pair, which keeps it within the register budget of two work-groups per compute unit.
template <int TAPS, int CPT, bool MULTI, int KS>
__device__ __forceinline__ void patch_kernel_impl(const GemmArgs& a, const PatchGeom& g, int pairs_per_wg) {
  RMSMP_PHASE(0);
  // Work-group id -> (pixel tile bx, row block by).  Consecutive ids go to different XCDs, each
  // with its own L2, so the gy work-groups that read the same input patch get ids that are equal
  // modulo 8 and follow each other on that XCD: the patch comes out of memory once, not gy
  // times.  The grid is padded to a multiple of 8 pixel tiles; the extra work-groups leave.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int by = slot % g.gy;
  const int bx = (slot / g.gy) * 8 + xcd;
  if (bx >= g.gx) return;
  EpArgs ea = pin_epilogue_args(a);
  ea.stamps = PHASE_LDS_BYTES != 0;
  RMSMP_PHASE(14);
  const int n_pairs = (a.w.n_tiles + 1) / 2;
  const int pair_lo = MULTI ? by * pairs_per_wg : by;
  const int pair_hi = MULTI ? min(pair_lo + pairs_per_wg, n_pairs) : pair_lo + 1;
  PatchState ps;
  ps.n0 = bx * pt_bn(KS);
  PairLoads pl;
  pl.T0 = pl.T1 = make_uint4(0, 0, 0, 0);
  int pi = pair_lo;
  bool first = true;
#pragma unroll 1
  while (pi < pair_hi) {
    const int k0 = tile_ref(a.w, pi).kind, k1 = tile_ref(a.w, a.w.n_tiles - 1 - pi).kind;
#define RMSMP_BODY(K0, K1) \
  if (k0 == K0 && k1 == K1) pi = patch_body<TAPS, CPT, K0, K1, MULTI, KS>(a, ea, g, ps, pl, first, pi, pair_hi);
    RMSMP_BODY(TILE_NIB_SHIFT, TILE_NIB_SHIFT)
    else RMSMP_BODY(TILE_NIB_SHIFT, TILE_NIB_LUT)
    else RMSMP_BODY(TILE_NIB_SHIFT, TILE_I8)
    else RMSMP_BODY(TILE_NIB_LUT, TILE_NIB_LUT)
    else RMSMP_BODY(TILE_NIB_LUT, TILE_I8)
    else RMSMP_BODY(TILE_I8, TILE_I8)
    else break;  // classes are sorted, so no other combination exists
#undef RMSMP_BODY
    first = false;
    if (!MULTI) break;
  }
  RMSMP_PHASE_FLUSH();
}

template <int TAPS, int CPT>
__global__ __launch_bounds__(PT_THREADS, 2) void conv_patch_kernel(GemmArgs a, PatchGeom g) {
  patch_kernel_impl<TAPS, CPT, false, 2>(a, g, 1);
}

// The same with four waves per output block (64 pixels per work-group) for small grids.
template <int TAPS, int CPT>
__global__ __launch_bounds__(PT_THREADS, 2) void conv_patch_split4_kernel(GemmArgs a, PatchGeom g) {
  patch_kernel_impl<TAPS, CPT, false, 4>(a, g, 1);
}

template <int TAPS, int CPT>
__global__ __launch_bounds__(PT_THREADS) void conv_patch_multi_kernel(GemmArgs a, PatchGeom g, int pairs_per_wg) {
  patch_kernel_impl<TAPS, CPT, true, 2>(a, g, pairs_per_wg);
}

static uint32_t div_magic(int64_t d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + (uint64_t)d - 1) / (uint64_t)d); }

// Channel counts (in K steps of 32) the LDS-resident kernel is instantiated for.
static bool patch_cpt_supported(int taps, int cpt) {
  if (taps == 9) return cpt == 2 || cpt == 4 || cpt == 8 || cpt == 16;
  return cpt == 2 || cpt == 4 || cpt == 8 || cpt == 16 || cpt == 24;
}

// How the LDS-resident kernel is launched.
struct PatchPlan {
  GemmArgs a;  // the argument block (a plain GEMM becomes a 1x1 convolution over N single-pixel images)
  PatchGeom g;
  size_t lds = 0;
  unsigned blocks = 0;
  int ks = 2;            // K split
  int pairs_per_wg = 1;  // > 1: the multi-pair kernel
};

// Geometry checks for the LDS-resident kernel; fills the plan when it applies.
static bool patch_kernel_applies(const GemmArgs& a0, PatchPlan* plan) {
  if (a0.ep.act_bits != 4) return false;
  GemmArgs a = a0;
  if (!a.conv) {
    if (a.K % (2 * KSTEP) != 0 || a.K > 1024 || a.N >= ((int64_t)1 << 30)) return false;
    a.conv = 1;
    a.d = rmsmp_conv_desc{(int32_t)a.N, (int32_t)a.K, 1, 1, 1, 1, 1, 0};
    a.OH = a.OW = 1;
  }
  const int taps = a.d.KH * a.d.KW;
  if (!(taps == 1 || (a.d.KH == 3 && a.d.KW == 3))) return false;
  // a strided 1x1 layer would stage stride^2 times the pixels it uses: the general kernel gathers instead
  if (taps == 1 && a.d.stride > 1) return false;
  const int cpt = a.d.C / KSTEP;
  if (a.d.C % KSTEP != 0 || !patch_cpt_supported(taps, cpt)) return false;
  if (a.w.nks != taps * cpt) return false;
  // The flattened input index of tap (0,0) must grow with the output pixel number, also across
  // output rows and images, so that a tile's pixels lie in one contiguous run of the input.
  const int64_t S = a.d.stride;
  const int64_t row_extra = S * ((int64_t)a.d.W - a.OW);                   // extra advance at an output-row boundary
  const int64_t img_extra = (int64_t)a.d.W * ((int64_t)a.d.H - S * a.OH);  // and, on top, at an image boundary
  if (row_extra < 0 || row_extra + img_extra < 0) return false;
  const int64_t hw = (int64_t)a.OH * a.OW, in_px = (int64_t)a.d.B * a.d.H * a.d.W;
  const int rs = a.d.C + 16;
  // widest run of flattened input pixels a tile of bn output pixels touches
  auto span_of = [&](int64_t bn) -> int64_t {
    const int64_t rows_crossed = (bn + a.OW - 1) / a.OW + 1, imgs_crossed = (bn + hw - 1) / hw + 1;
    return (bn - 1) * S + 1 + (int64_t)(a.d.KH - 1) * a.d.W + (a.d.KW - 1) + rows_crossed * row_extra +
           imgs_crossed * (img_extra > 0 ? img_extra : 0);
  };
  const int n_pairs = (a.w.n_tiles + 1) / 2;
  // Four waves per output block when the grid would otherwise leave more than half of the
  // compute units idle (and a tap holds a multiple of four K steps): twice the work-groups, each
  // with half the K loop.  With both splits able to fill the chip the two-way split is faster
  // (measured): less partial-sum traffic, and two work-groups on a compute unit mostly compete
  // for the same vector-instruction issue slots.
  int ks = 2;
  if (cpt % 4 == 0 && (a.N + pt_bn(2) - 1) / pt_bn(2) * n_pairs <= 128) ks = 4;
  const int64_t bn = pt_bn(ks);
  const int64_t span = span_of(bn);
  // 32-bit pixel arithmetic and exact one-multiply division in the kernel
  if ((a.N + bn) * hw >= ((int64_t)1 << 32) || in_px * (a.d.C / 2) >= ((int64_t)1 << 40)) return false;
  if (in_px + span >= ((int64_t)1 << 31) / rs) return false;
  const size_t need = (size_t)(span + 1) * rs;  // patch + zero-point row
  // One tile pair per work-group (the exchange buffer overlays the patch) unless the patch is so
  // large that only one work-group fits a compute unit anyway: then a work-group keeps its patch
  // and runs through several pairs, as long as the grid still fills the chip.
  const size_t xch = (size_t)pt_xch_bytes(ks);
  const size_t lds_single = PHASE_LDS_BYTES + PT_META_BYTES + (need > xch ? need : xch);
  const size_t lds_multi = PHASE_LDS_BYTES + PT_META_BYTES + xch + need;
  if (lds_single > 160 * 1024) return false;
  const int64_t gx = (a.N + bn - 1) / bn;
  int64_t ppw = 1;
  if (ks == 2 && lds_single > 80 * 1024 && lds_multi <= 160 * 1024) {
    ppw = gx * n_pairs / 256;
    ppw = ppw < 1 ? 1 : ppw > n_pairs ? n_pairs : ppw;
  }
  const int gy = (int)((n_pairs + ppw - 1) / ppw);
  ppw = (n_pairs + gy - 1) / gy;
  if ((gx + 7) / 8 * 8 * gy > 0x7fffffff) return false;
  plan->a = a;
  plan->g.gx = (int)gx;
  plan->g.gy = gy;
  plan->g.row_stride = rs;
  plan->g.patch_rows = (int)span;
  plan->g.magic_hw = div_magic(hw);
  plan->g.magic_ow = div_magic(a.OW);
  plan->lds = ppw == 1 ? lds_single : lds_multi;
  plan->blocks = (unsigned)((gx + 7) / 8 * 8 * gy);
  plan->ks = ks;
  plan->pairs_per_wg = (int)ppw;
  return true;
}

// Dynamic LDS above 64 KiB must be allowed per kernel once (per device); remember what was set.
template <int TAPS, int CPT>
static int launch_patch_t(const PatchPlan& p, hipStream_t s) {
  static bool allowed[64] = {false};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= 64) return (int)hipErrorInvalidDevice;
  if (!allowed[dev]) {
    e = hipFuncSetAttribute((const void*)conv_patch_kernel<TAPS, CPT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            160 * 1024);
    if (e != hipSuccess) return (int)e;
    e = hipFuncSetAttribute((const void*)conv_patch_multi_kernel<TAPS, CPT>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return (int)e;
    if constexpr (CPT % 4 == 0) {
      e = hipFuncSetAttribute((const void*)conv_patch_split4_kernel<TAPS, CPT>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e != hipSuccess) return (int)e;
    }
    allowed[dev] = true;
  }
  const dim3 grid(p.blocks), block(PT_THREADS);
  if (p.pairs_per_wg > 1) {
    hipLaunchKernelGGL((conv_patch_multi_kernel<TAPS, CPT>), grid, block, p.lds, s, p.a, p.g, p.pairs_per_wg);
  } else if (p.ks == 4) {
    if constexpr (CPT % 4 == 0)
      hipLaunchKernelGGL((conv_patch_split4_kernel<TAPS, CPT>), grid, block, p.lds, s, p.a, p.g);
    else
      return (int)hipErrorInvalidValue;
  } else {
    hipLaunchKernelGGL((conv_patch_kernel<TAPS, CPT>), grid, block, p.lds, s, p.a, p.g);
  }
  return (int)hipGetLastError();
}

static int launch_patch(const PatchPlan& p, hipStream_t s) {
  const int taps = p.a.d.KH * p.a.d.KW;
  const int cpt = p.a.d.C / KSTEP;
#define RMSMP_PATCH_CASE(TP, CP) \
  if (taps == TP && cpt == CP) return launch_patch_t<TP, CP>(p, s);
  RMSMP_PATCH_CASE(9, 2)
  RMSMP_PATCH_CASE(9, 4)
  RMSMP_PATCH_CASE(9, 8)
  RMSMP_PATCH_CASE(9, 16)
  RMSMP_PATCH_CASE(1, 2)
  RMSMP_PATCH_CASE(1, 4)
  RMSMP_PATCH_CASE(1, 8)
  RMSMP_PATCH_CASE(1, 16)
  RMSMP_PATCH_CASE(1, 24)
#undef RMSMP_PATCH_CASE
  return (int)hipErrorInvalidValue;
}

// ---------------------------------------------------------------- skinny GEMM (N <= 64)
//
// A handful of activation columns against a large weight matrix moves every packed weight byte
// once and does almost no arithmetic: the kernel is a weight stream at memory speed.  One
// work-group per weight tile, eight waves; wave w takes one eighth of K.  It issues all of its
// weight reads (one fully coalesced 512-byte / 1-KiB fragment per K step) before touching any of
// them, so a work-group keeps its whole 32-row slab in flight; its slice of the activations goes
// through a private LDS region (packed, decoded per fragment).  The eight partial sums are added
// through LDS and finished by the usual epilogue.
constexpr int SK_THREADS = 512;
constexpr int SK_WAVES = 8;
constexpr int SK_CHUNK = 16;  // K steps whose loads are in flight together per wave

template <int KIND, int NB>
__device__ __forceinline__ void skinny_body(const GemmArgs& a, uint8_t* smem, const TileRef& tr, int mt) {
  const EpArgs ea = pin_epilogue_args(a);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  constexpr int FRAG = KIND == TILE_I8 ? 16 : 8;
  constexpr int ROWS = 32 * NB;
  const int nks = a.w.nks;
  const int S = (nks + SK_WAVES - 1) / SK_WAVES;  // K steps per wave
  const int ks0 = wave * S;
  const uint8_t* wbase = a.w.blob + tr.blob_off;
  const uint32_t wl = (uint32_t)lane * FRAG;
  uint4 T = make_uint4(0, 0, 0, 0);
  if (KIND == TILE_NIB_LUT) T = *(const uint4*)(a.w.p_lut + ((int64_t)mt * TILE_M + tile_row_goff(lane & 31)) * 4);
  const uint8_t* X = (const uint8_t*)a.X;
  const int64_t ldx = a.K / 2;
  const int x_stride = SK_CHUNK * 16 + 8;  // LDS bytes per activation row of a chunk (padded)
  uint8_t* xs = smem + wave * (ROWS * x_stride);

  v16i acc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0;

#pragma unroll 1
  for (int c0 = 0; c0 < S; c0 += SK_CHUNK) {
    // all weight fragments of the chunk first ...
    typename RawFrag<KIND>::type raw[SK_CHUNK];
#pragma unroll
    for (int u = 0; u < SK_CHUNK; ++u) {
      int ks = ks0 + c0 + u;
      ks = ks < nks ? ks : nks - 1;
      raw[u] = load_raw<KIND>(wbase + (int64_t)ks * (LANES * FRAG), wl);
    }
    // ... then this wave's slice of the activations: ROWS rows x (SK_CHUNK*16) packed bytes
    {
      const int64_t col0 = (int64_t)(ks0 + c0) * 16;  // byte offset inside an activation row
#pragma unroll
      for (int i = 0; i < ROWS * SK_CHUNK / LANES; ++i) {
        const int pidx = i * LANES + lane;
        const int row = pidx / SK_CHUNK, piece = pidx % SK_CHUNK;
        const int64_t n = row < (int)a.N ? row : (int)a.N - 1;  // rows past N repeat the last one; never stored
        int64_t cb = col0 + piece * 16;
        cb = cb + 16 <= ldx ? cb : ldx - 16;  // past the end of K: any data, its weights are zero
        const uint4 w = *(const uint4*)(X + n * ldx + cb);
        *(uint2*)(xs + row * x_stride + piece * 16) = make_uint2(w.x, w.y);
        *(uint2*)(xs + row * x_stride + piece * 16 + 8) = make_uint2(w.z, w.w);
      }
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's LDS writes have landed (region is private)
#pragma unroll
    for (int u = 0; u < SK_CHUNK; ++u) {
      const int ks = ks0 + c0 + u;
      if (c0 + u < S && ks < nks) {
        const v4i av = decode_raw<KIND>(raw[u], T);
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          const uint2 xw = *(const uint2*)(xs + (32 * j + (lane & 31)) * x_stride + u * 16 + (lane >> 5) * 8);
          acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, decode_act_u4(xw), acc[j], 0, 0, 0);
        }
      }
    }
  }

  // ---- add the eight partial sums: wave j (< NB) finishes pixel block j
  __syncthreads();
  {
    int* dst = (int*)smem + wave * (NB * 16 * LANES);
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *(v4i*)(dst + j * (16 * LANES) + q * (4 * LANES) + lane * 4) =
            (v4i){acc[j][4 * q], acc[j][4 * q + 1], acc[j][4 * q + 2], acc[j][4 * q + 3]};
  }
  __syncthreads();
  if (wave >= NB) return;
  v16i sum[1];
#pragma unroll
  for (int r = 0; r < 16; ++r) sum[0][r] = 0;
#pragma unroll 1
  for (int w = 0; w < SK_WAVES; ++w) {
    const int* src = (const int*)smem + w * (NB * 16 * LANES) + wave * (16 * LANES);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const v4i got = *(const v4i*)(src + q * (4 * LANES) + lane * 4);
      sum[0][4 * q] += got.x;
      sum[0][4 * q + 1] += got.y;
      sum[0][4 * q + 2] += got.z;
      sum[0][4 * q + 3] += got.w;
    }
  }
  RowMeta rm;
  load_row_meta(a.w, mt, lane, rm);
  const int64_t ncol[1] = {32 * wave + (lane & 31)};
  finish_tiles<1>(ea, KIND, sum, rm, lane_rows(tr.nvalid, lane), ncol);
}

template <int NB>
__global__ __launch_bounds__(SK_THREADS) void gemm_skinny_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
  const int mt = blockIdx.x;
  const TileRef tr = tile_ref(a.w, mt);
  if (tr.kind == TILE_NIB_SHIFT)
    skinny_body<TILE_NIB_SHIFT, NB>(a, smem_raw, tr, mt);
  else if (tr.kind == TILE_NIB_LUT)
    skinny_body<TILE_NIB_LUT, NB>(a, smem_raw, tr, mt);
  else
    skinny_body<TILE_I8, NB>(a, smem_raw, tr, mt);
}

static bool skinny_applies(const GemmArgs& a) {
  return !a.conv && a.ep.act_bits == 4 && a.N <= 64 && a.K % 64 == 0 && a.K >= 512;
}

template <int NB>
static int launch_skinny_t(const GemmArgs& a, hipStream_t s) {
  const size_t xs = (size_t)SK_WAVES * 32 * NB * (SK_CHUNK * 16 + 8);
  const size_t xch = (size_t)SK_WAVES * NB * 16 * LANES * 4;
  const size_t lds = xs > xch ? xs : xch;
  static bool allowed[64] = {false};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= 64) return (int)hipErrorInvalidDevice;
  if (!allowed[dev]) {
    e = hipFuncSetAttribute((const void*)gemm_skinny_kernel<NB>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return (int)e;
    allowed[dev] = true;
  }
  hipLaunchKernelGGL(gemm_skinny_kernel<NB>, dim3((unsigned)a.w.n_tiles), dim3(SK_THREADS), lds, s, a);
  return (int)hipGetLastError();
}

// ---------------------------------------------------------------- small-channel convolution
//
// A network's first layer: 8-bit activations, at most four input channels, a square filter of up
// to 8x8, any stride.  Its lowered matrix would be by far the largest tensor of the layer (K =
// 147 bytes per output pixel against 3 bytes per input pixel), so nothing is lowered: a
// work-group stages the input pixels of an 8 x 16 tile of output pixels in LDS, each pixel padded
// to four bytes, and reads B fragments straight from there.  The weights are stored with one K
// step per filter row (KLayout K_FILTER_ROWS), so the 16 bytes a lane needs for K step kh are
// four consecutive staged pixels of input row oh*stride - pad + kh.
//
// Four waves; wave w owns output rows 2w, 2w+1 of the tile (32 pixels) and goes through the
// layer's weight tiles one at a time.  A lane's B fragments (one per filter row) are read from
// LDS once and kept; per weight tile it then loads KH weight fragments, issues KH MFMAs and runs
// the epilogue, with the row metadata of all tiles staged in LDS at the start.  Few registers,
// so several work-groups share a compute unit and hide each other's memory latency.
constexpr int CR_TH = 8, CR_TW = 16;
constexpr int CR_MAX_TILES = 64;  // row metadata of all tiles sits in LDS (512 bytes per tile)

// KHW: filter height = width as a compile-time constant (3, 5, 7), or 0 for any size up to 8.
template <int KHW_T>
__global__ __launch_bounds__(256, 3) void conv_rows_kernel(GemmArgs a, int tiles_w, int tiles_h) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
  const EpArgs ea = pin_epilogue_args(a);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  constexpr int KMAX = KHW_T ? KHW_T : 8;
  const int KHW = KHW_T ? KHW_T : a.d.KH;
  const int S = a.d.stride, C = a.d.C, H = a.d.H, W = a.d.W;
  int blk = blockIdx.x;
  const int tw = blk % tiles_w;
  blk /= tiles_w;
  const int th = blk % tiles_h;
  const int b = blk / tiles_h;
  const int oh0 = th * CR_TH, ow0 = tw * CR_TW;
  const int PH = S * (CR_TH - 1) + KHW;  // staged rows
  const int PW = S * (CR_TW - 1) + 8;    // staged pixels per row (a fragment reads 8 pixels from its first)
  const int ih0 = oh0 * S - a.d.pad, iw0 = ow0 * S - a.d.pad;
  int* const meta = (int*)(smem_raw + (size_t)PH * PW * 4);  // [tile][field][32 rows]

  // ---- stage the input pixels, four bytes each (missing channels 0, out-of-image = zero point)
  {
    const uint8_t* X = (const uint8_t*)a.X;
    const uint32_t z = (uint32_t)a.ep.act_zero_point & 255u;
    uint32_t zfill = 0u;
    for (int c = 0; c < C; ++c) zfill |= z << (8 * c);
    for (int idx = tid; idx < PH * PW; idx += 256) {
      const int py = idx / PW, px = idx - py * PW;
      const int ih = ih0 + py, iw = iw0 + px;
      uint32_t v = zfill;
      if (ih >= 0 && ih < H && iw >= 0 && iw < W) {
        const uint8_t* src = X + (((int64_t)b * H + ih) * W + iw) * C;
        v = 0u;
        for (int c = 0; c < C; ++c) v |= (uint32_t)src[c] << (8 * c);
      }
      ((uint32_t*)smem_raw)[idx] = v;
    }
    for (int idx = tid; idx < a.w.n_tiles * TILE_M; idx += 256) {
      const int4 m = ((const int4*)a.w.p_meta)[idx];
      int* dst = meta + (idx / TILE_M) * (4 * TILE_M) + (idx % TILE_M);
      dst[0] = m.x;
      dst[TILE_M] = m.y;
      dst[2 * TILE_M] = m.z;
      dst[3 * TILE_M] = m.w;
    }
  }
  __syncthreads();

  // this lane's output pixel and its B fragments: four consecutive staged pixels per filter row
  const int pr = 2 * wave + ((lane & 31) >> 4), pc = lane & 15;
  const int oh = oh0 + pr, ow = ow0 + pc;
  const bool px_ok = oh < a.OH && ow < a.OW;
  const int64_t n = px_ok ? ((int64_t)b * a.OH + oh) * a.OW + ow : a.N;  // a.N = no store
  const uint32_t* sp = (const uint32_t*)smem_raw + (pr * S) * PW + pc * S + 4 * (lane >> 5);
  v4i bf[KMAX];
#pragma unroll
  for (int kh = 0; kh < KMAX; ++kh) {
    const uint32_t* q = sp + (kh < KHW ? kh : 0) * PW;
    bf[kh] = reorder_act_i8(make_uint4(q[0], q[1], q[2], q[3]));
  }

#pragma unroll 1
  for (int mt = 0; mt < a.w.n_tiles; ++mt) {
    const TileRef tr = tile_ref(a.w, mt);
    const uint8_t* wp = a.w.blob + tr.blob_off;
    v4i af[KMAX];
    // filter rows beyond KHW (generic build only) repeat row 0 and are not multiplied
    if (tr.kind == TILE_I8) {
#pragma unroll
      for (int kh = 0; kh < KMAX; ++kh)
        af[kh] = decode_raw<TILE_I8>(load_raw<TILE_I8>(wp, (uint32_t)((kh < KHW ? kh : 0) * LANES + lane) * 16),
                                     make_uint4(0, 0, 0, 0));
    } else if (tr.kind == TILE_NIB_SHIFT) {
#pragma unroll
      for (int kh = 0; kh < KMAX; ++kh)
        af[kh] = decode_raw<TILE_NIB_SHIFT>(
            load_raw<TILE_NIB_SHIFT>(wp, (uint32_t)((kh < KHW ? kh : 0) * LANES + lane) * 8), make_uint4(0, 0, 0, 0));
    } else {
      const uint4 T = *(const uint4*)(a.w.p_lut + ((int64_t)mt * TILE_M + tile_row_goff(lane & 31)) * 4);
#pragma unroll
      for (int kh = 0; kh < KMAX; ++kh)
        af[kh] = decode_raw<TILE_NIB_LUT>(load_raw<TILE_NIB_LUT>(wp, (uint32_t)((kh < KHW ? kh : 0) * LANES + lane) * 8), T);
    }
    v16i acc[1];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][r] = 0;
#pragma unroll
    for (int kh = 0; kh < KMAX; ++kh)
      if (kh < KHW) acc[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[kh], bf[kh], acc[0], 0, 0, 0);
    RowMetaLds rm;
    rm.base = (const int*)__builtin_assume_aligned(meta + mt * (4 * TILE_M) + 16 * (lane >> 5), 64);
    rm.rows = TILE_M;
    const int64_t ncol[1] = {n};
    finish_tiles<1>(ea, tr.kind, acc, rm, lane_rows(tr.nvalid, lane), ncol);
  }
}

static bool conv_rows_applies(const GemmArgs& a) {
  return a.conv && a.w.k_layout == K_FILTER_ROWS && a.ep.act_bits == 8 && a.d.KH == a.d.KW && a.d.KW <= 8 && a.d.C <= 4 &&
         a.w.nks >= a.d.KH && a.d.stride <= 8 && a.w.n_tiles <= CR_MAX_TILES;
}

static int launch_conv_rows(const GemmArgs& a, hipStream_t s) {
  const int tiles_w = (a.OW + CR_TW - 1) / CR_TW, tiles_h = (a.OH + CR_TH - 1) / CR_TH;
  const int64_t blocks = (int64_t)a.d.B * tiles_w * tiles_h;
  if (blocks > 0x7fffffff) return (int)hipErrorInvalidValue;
  const int PH = a.d.stride * (CR_TH - 1) + a.d.KH, PW = a.d.stride * (CR_TW - 1) + 8;
  const size_t lds = (size_t)PH * PW * 4 + (size_t)a.w.n_tiles * TILE_M * 16;  // at most 63 KiB
  const dim3 grid((unsigned)blocks), block(256);
  switch (a.d.KH) {
    case 3: hipLaunchKernelGGL(conv_rows_kernel<3>, grid, block, lds, s, a, tiles_w, tiles_h); break;
    case 5: hipLaunchKernelGGL(conv_rows_kernel<5>, grid, block, lds, s, a, tiles_w, tiles_h); break;
    case 7: hipLaunchKernelGGL(conv_rows_kernel<7>, grid, block, lds, s, a, tiles_w, tiles_h); break;
    default: hipLaunchKernelGGL(conv_rows_kernel<0>, grid, block, lds, s, a, tiles_w, tiles_h); break;
  }
  return (int)hipGetLastError();
}

int launch_gemm(const GemmArgs& a, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  if (a.N <= 0) return 0;
  if (conv_rows_applies(a)) return launch_conv_rows(a, s);
  if (!a.conv && skinny_applies(a)) return a.N <= 32 ? launch_skinny_t<1>(a, s) : launch_skinny_t<2>(a, s);
  {
    PatchPlan plan;
    if (patch_kernel_applies(a, &plan)) return launch_patch(plan, s);
  }
  if (a.conv) return a.ep.act_bits == 4 ? launch_general<4, true, true>(a, s) : launch_general<8, true, true>(a, s);
  const bool vec = (a.K % 16) == 0;
  if (a.ep.act_bits == 4) return vec ? launch_general<4, false, true>(a, s) : launch_general<4, false, false>(a, s);
  return vec ? launch_general<8, false, true>(a, s) : launch_general<8, false, false>(a, s);
}

// ---------------------------------------------------------------- explicit im2col
//
// Fallback for layers whose channel count is not a multiple of 16: writes the lowered matrix
// [N][Kpad] in the K order the weights are stored in (either KLayout).
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
    int kh, kw, cc;
    if (a.k_layout == K_FILTER_ROWS) {
      kh = (int)(kk / KSTEP);
      const int r = (int)(kk - (int64_t)kh * KSTEP);
      kw = r / 4;
      cc = r - 4 * kw;
      if (kh >= a.d.KH || kw >= a.d.KW || cc >= a.d.C) return 0u;  // the weight there is zero
    } else {
      if (kk >= a.K) return 0u;
      const int tap = (int)(kk / a.d.C);
      cc = (int)(kk - (int64_t)tap * a.d.C);
      kh = tap / a.d.KW;
      kw = tap - kh * a.d.KW;
    }
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
