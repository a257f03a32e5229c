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

#include "device_common.h"

namespace rmsmp {

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
typedef unsigned sk_v2w __attribute__((ext_vector_type(2)));
typedef unsigned sk_v4w __attribute__((ext_vector_type(4)));

// What a wave needs before it can issue its weight and activation reads, fetched from the kernel
// arguments in one go at the start of the kernel.
struct SkinnyFirst {
  const uint8_t* blob;
  const void* X;
  const uint32_t* p_lut;
  int nks, ldx, N;
};

template <int KIND, int NB>
__device__ __forceinline__ void skinny_body(const SkinnyFirst& f, const GemmArgs& a, uint8_t* smem, const TileRef& tr, int mt) {
  RMSMP_REG_STAMPS_DECLARE();
  RMSMP_REG_STAMP(0);
  EpArgs ea{};  // fetched once the first reads are on their way (the argument block comes from memory)
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  constexpr int FRAG = KIND == TILE_I8 ? 16 : 8;
  constexpr int ROWS = 32 * NB;
  const int nks = f.nks;
  const bool few = f.N <= ROWS / 2;  // at most half of the columns exist: leave the other activation reads out
  const int S = (nks + SK_WAVES - 1) / SK_WAVES;  // K steps per wave
  const int ks0 = wave * S;
  // Weights and activations are read through buffer descriptors: the K-step offset of a weight
  // read and the column offset of an activation read are scalar, the per-lane offsets are formed
  // once, and a read past the end returns zeros (whose products are never used), so the reads at
  // the start of the kernel -- which run at the speed of instruction fetch, one wave of a SIMD
  // after the other -- cost one instruction each instead of a 64-bit address each.
  const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc((void*)(f.blob + tr.blob_off), 0, nks * (LANES * FRAG), 0x00020000);
  const uint32_t wl = (uint32_t)lane * FRAG;
  uint4 T = make_uint4(0, 0, 0, 0);
  if (KIND == TILE_NIB_LUT) T = *(const uint4*)(f.p_lut + ((int64_t)mt * TILE_M + tile_row_goff(lane & 31)) * 4);
  const int ldx = f.ldx;
  const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc((void*)f.X, 0, f.N * ldx, 0x00020000);
  const int x_stride = SK_CHUNK * 16 + 8;  // LDS bytes per activation row of a chunk (padded)
  uint8_t* xs = smem + wave * (ROWS * x_stride);

  v16i acc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0;

#pragma unroll 1
  for (int c0 = 0; c0 < S; c0 += SK_CHUNK) {
    // All weight fragments of the chunk first -- they come from memory and their addresses need next
    // to no arithmetic, and the code that runs once at the start of a kernel runs at the speed of
    // instruction fetch, so every instruction in front of these reads delays them -- then this
    // wave's slice of the activations (ROWS rows x SK_CHUNK*16 packed bytes, a few KB from the cache).
    typename RawFrag<KIND>::type raw[SK_CHUNK];
#pragma unroll
    for (int u = 0; u < SK_CHUNK; ++u) {
      const int soff = (ks0 + c0 + u) * (LANES * FRAG);  // past the end of the tile: zeros
      if constexpr (KIND == TILE_I8) {
        const sk_v4w w = __builtin_amdgcn_raw_buffer_load_b128(wrs, (int)wl, soff, 0);
        raw[u] = make_uint4(w.x, w.y, w.z, w.w);
      } else {
        const sk_v2w w = __builtin_amdgcn_raw_buffer_load_b64(wrs, (int)wl, soff, 0);
        raw[u] = make_uint2(w.x, w.y);
      }
    }
    constexpr int XI = ROWS * SK_CHUNK / LANES;
    static_assert(LANES % SK_CHUNK == 0, "a lane keeps its piece number over the reads of a chunk");
    uint4 xw[XI];
    {
      const int col0 = (ks0 + c0) * 16;  // byte offset inside an activation row (scalar)
      const int piece = lane % SK_CHUNK, row0 = lane / SK_CHUNK;
      const int n_last = f.N - 1;
      // A read covers LANES / SK_CHUNK rows.  With fewer than ROWS columns the reads whose rows all
      // lie past N are left out (their LDS rows keep whatever they hold: columns past N are computed
      // and never stored); with all of them the reads are unconditional, in one batch.
      auto read_x = [&](auto few_tag) {
        constexpr bool FEW = decltype(few_tag)::value;
#pragma unroll
        for (int i = 0; i < XI; ++i) {
          if (FEW && i * (LANES / SK_CHUNK) > n_last) continue;
          const int row = i * (LANES / SK_CHUNK) + row0;
          const int n = row < n_last ? row : n_last;
          // (past the end of K: whatever follows in the tensor or zeros, its weights are zero)
          const sk_v4w w = __builtin_amdgcn_raw_buffer_load_b128(xrs, n * ldx + piece * 16, col0, 0);
          xw[i] = make_uint4(w.x, w.y, w.z, w.w);
        }
      };
      if (few)
        read_x(std::true_type{});
      else
        read_x(std::false_type{});
    }
    if (c0 == 0) ea = pin_epilogue_args(a);
    RMSMP_REG_STAMP(1);
#pragma unroll
    for (int i = 0; i < XI; ++i) {
      if (few && i * (LANES / SK_CHUNK) > f.N - 1) continue;
      const int pidx = i * LANES + lane;
      const int row = pidx / SK_CHUNK, piece = pidx % SK_CHUNK;
      *(uint2*)(xs + row * x_stride + piece * 16) = make_uint2(xw[i].x, xw[i].y);
      *(uint2*)(xs + row * x_stride + piece * 16 + 8) = make_uint2(xw[i].z, xw[i].w);
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's LDS writes have landed (region is private)
    RMSMP_REG_STAMP(2);
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

  RMSMP_REG_STAMP(3);
  // The usual case of this kernel -- fp32 output, no bias, a full weight tile, an output small
  // enough for 32-bit byte offsets -- is finished by all eight waves together: wave w adds up
  // accumulator registers 2w and 2w+1 of the eight partial sums (rows 2w, 2w+1 of either half of
  // the tile), scales them and stores them.  The code after the last barrier runs once, at the speed
  // of instruction fetch, so one wave finishing 16 values per lane (the general path below) takes
  // eight times as long as eight waves finishing two each.  Same arithmetic, same order.
  const bool fast = ea.out_kind == 1 && ea.bias == nullptr && tr.nvalid == TILE_M && ea.M * ea.N < ((int64_t)1 << 30);
  // The general path fetches its row metadata now, behind the barriers and the reduction: at the
  // end it would be one more memory round trip in front of the stores.  (Not earlier: a load under
  // a wave-dependent branch makes the compiler drain every outstanding load where the branches
  // join, and up there that would be in front of the weight reads.)
  RowMeta rm;
  int4 my_rows[2] = {make_int4(0, 0, 0, 0), make_int4(0, 0, 0, 0)};
  if (fast) {  // (fetched up front, behind the weight reads, these two reads measured no better)
    const int4* src = (const int4*)a.w.p_meta + (int64_t)mt * TILE_M + 16 * (lane >> 5) + 2 * wave;
    my_rows[0] = src[0];
    my_rows[1] = src[1];
  } else if (wave < NB) {
    load_row_meta(a.w, mt, lane, rm);
  }
  // ---- add the eight partial sums
  __syncthreads();
  RMSMP_REG_STAMP(4);
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
  RMSMP_REG_STAMP(5);
  if (fast) {
    const __amdgpu_buffer_rsrc_t yr = __builtin_amdgcn_make_buffer_rsrc(ea.Y, 0, (int)(ea.M * ea.N * 4), 0x00020000);
    const int N = (int)ea.N;
    const bool x16 = KIND == TILE_NIB_SHIFT;
    const int zs = x16 ? 16 * ea.zp : ea.zp;
    const float fold = x16 ? 0.0625f : 1.0f;
    const float floor_y = ea.relu ? 0.0f : -__builtin_inff();
    const float m0 = __fmul_rn(__fmul_rn(__int_as_float(my_rows[0].x), ea.act_scale), fold);
    const float m1 = __fmul_rn(__fmul_rn(__int_as_float(my_rows[1].x), ea.act_scale), fold);
    // registers 2w, 2w+1 sit in 16-byte group w/2 of a partial sum, at its elements (2w)%4, (2w)%4+1
    const int* part = (const int*)smem + (wave >> 1) * (4 * LANES) + lane * 4 + ((2 * wave) & 3);
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      int s0 = 0, s1 = 0;
#pragma unroll
      for (int w = 0; w < SK_WAVES; ++w) {
        const int2 got = *(const int2*)(part + w * (NB * 16 * LANES) + j * (16 * LANES));
        s0 += got.x;
        s1 += got.y;
      }
      const float y0 = fmaxf(__fmul_rn((float)(s0 - zs * my_rows[0].y), m0), floor_y);
      const float y1 = fmaxf(__fmul_rn((float)(s1 - zs * my_rows[1].y), m1), floor_y);
      const int n = 32 * j + (lane & 31);
      if (n < N) {
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(y0), yr, (__mul24(my_rows[0].z, N) + n) * 4, 0, 0);
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(y1), yr, (__mul24(my_rows[1].z, N) + n) * 4, 0, 0);
      }
    }
    RMSMP_REG_STAMP(7);
    RMSMP_REG_STAMPS_FLUSH();
    return;
  }
  if (wave >= NB) {
    RMSMP_REG_STAMPS_FLUSH();
    return;
  }
  v16i sum[1];
#pragma unroll
  for (int r = 0; r < 16; ++r) sum[0][r] = 0;
  // (four waves' parts in flight at a time: read one after the other, the eight LDS round trips add up)
#pragma unroll 4
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
  RMSMP_REG_STAMP(6);
  const int64_t ncol[1] = {32 * wave + (lane & 31)};
  finish_tiles<1>(ea, KIND, sum, rm, lane_rows(tr.nvalid, lane), ncol);
  RMSMP_REG_STAMP(7);
  RMSMP_REG_STAMPS_FLUSH();
}

template <int NB>
__global__ __launch_bounds__(SK_THREADS) void gemm_skinny_kernel(GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
  // Every kernel argument the first reads need, asked for here: left to itself the compiler fetches
  // an argument where it is first used, which puts half a dozen dependent scalar-memory round trips
  // in front of the first weight read; this way they are one.  (Handing them over in registers at
  // wave launch -- kernel-argument preloading, which the wide kernels use -- delays the launch of
  // this kernel's eight waves per work-group by more than it saves: 6.7 -> 7.2 us.)
  asm volatile("" ::"s"(a.w.blob), "s"(a.w.p_lut), "s"(a.w.nks), "s"(a.w.class_tiles[0]), "s"(a.w.class_tiles[1]),
               "s"(a.w.class_rows[0]), "s"(a.w.class_rows[1]), "s"(a.w.class_rows[2]), "s"(a.K), "s"(a.N), "s"(a.X));
  const int mt = blockIdx.x;
  const TileRef tr = tile_ref(a.w, mt);
  const SkinnyFirst f{a.w.blob, a.X, a.w.p_lut, a.w.nks, (int)(a.K / 2), (int)a.N};
  if (tr.kind == TILE_NIB_SHIFT)
    skinny_body<TILE_NIB_SHIFT, NB>(f, a, smem_raw, tr, mt);
  else if (tr.kind == TILE_NIB_LUT)
    skinny_body<TILE_NIB_LUT, NB>(f, a, smem_raw, tr, mt);
  else
    skinny_body<TILE_I8, NB>(f, a, smem_raw, tr, mt);
}

static bool skinny_applies(const GemmArgs& a) {
  // (K below 2^24: the kernel's byte offsets into X and into a weight tile are 32-bit)
  return !a.conv && a.ep.act_bits == 4 && a.N <= 64 && a.K % 64 == 0 && a.K >= 512 && a.K < ((int64_t)1 << 24);
}

template <int NB>
static int launch_skinny_t(const GemmArgs& a, hipStream_t s) {
  const size_t xs = (size_t)SK_WAVES * 32 * NB * (SK_CHUNK * 16 + 8);
  const size_t xch = (size_t)SK_WAVES * NB * 16 * LANES * 4;
  const size_t lds = xs > xch ? xs : xch;
  static std::atomic<uint64_t> allowed{0};
  if (const int rc = allow_large_lds((const void*)gemm_skinny_kernel<NB>, allowed)) return rc;
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

int* forced_split() {
  static thread_local int split[4] = {0, 0, 0, 0};
  return split;
}
int allow_large_lds(const void* kernel, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= 64) return (int)hipErrorInvalidDevice;
  const uint64_t bit = (uint64_t)1 << dev;
  if (done.load(std::memory_order_acquire) & bit) return 0;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e != hipSuccess) return (int)e;
  done.fetch_or(bit, std::memory_order_release);
  return 0;
}
DispatchRecord& last_dispatch() {
  static thread_local DispatchRecord rec;
  return rec;
}

int launch_gemm(const GemmArgs& a, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  last_dispatch() = DispatchRecord{};
  if (a.N <= 0) return 0;
  {
    bool applied = false;
    const int rc = try_launch_conv_first(a, stream, &applied);
    if (applied) return rc;
  }
  if (conv_rows_applies(a)) {
    last_dispatch().kernel = 3;
    return launch_conv_rows(a, s);
  }
  if (!a.conv && skinny_applies(a)) {
    last_dispatch().kernel = 2;
    return a.N <= 32 ? launch_skinny_t<1>(a, s) : launch_skinny_t<2>(a, s);
  }
  {
    bool applied = false;
    const int rc = try_launch_wide(a, stream, &applied);
    if (applied) return rc;
  }
  last_dispatch().kernel = 1;
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
