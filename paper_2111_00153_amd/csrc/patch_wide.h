// LDS-resident implicit-im2col kernel of librmsmp (gfx950): 1x1 and 3x3 layers of any stride with
// 64 to 512 input channels, and plain GEMMs taken as 1x1 layers (K up to 768 in one piece, deeper
// ones staged in parts of 768 or 512 channels by the DEEP variant).
//
// The input pixels a work-group needs -- one contiguous run of the flattened NHWC tensor (strided
// 1x1 layers: exactly the pixels used, gathered) -- are read from memory once, decoded to int8
// and kept in LDS for all taps: implicit im2col, nothing is materialised, and a pixel is reused
// nine times from LDS.  Out-of-image taps read a row that holds the zero-point code.  Packed
// weights stream from global memory (buffer loads: descriptor and K offset in scalar registers)
// through a register ring a few K steps ahead of their use and are decoded in registers; the two
// weight tiles of a wave are tile y and tile (count-1-y), so a table-decoded (PoT) tile is paired
// with a cheap one whenever the layer has both.
//
// What the measurements asked for:
//  * The decode of a weight fragment is vector-ALU work (a vector instruction costs a lone wave
//    about six cycles of its SIMD, an MFMA 32; the two overlap, so a K step takes the larger sum).
//    A wave that owns 64 rows x 128 pixels (two weight fragments x four activation fragments,
//    eight MFMAs per K step) spends ~4 vector instructions per MFMA on a Fixed-4 + PoT-4 pair, at
//    64 pixels per wave ~8 (more than fit under one MFMA).  Both sizes exist (XB = 4 / 2): the
//    smaller one gives the grid more work-groups and lets three of them share a compute unit.
//  * The K loop is a real loop (one filter row, or one tap, per iteration) whose steps are cut in
//    sub-blocks "two MFMAs, a slice of next step's decode, one LDS read" that the scheduler may not
//    mix: every LDS read then has six MFMAs between issue and use, and the vector instructions sit
//    evenly in the shadow of the matrix pipe (40 cycles per MFMA in steady state, 32 = peak).
//  * A launch of the sizes at hand is one round of work-groups, so its time is one work-group's
//    critical path: every global read that needs only the kernel arguments is issued before
//    anything else (the patch before the code of the tile classes is even fetched), accumulator
//    zeroing and address arithmetic run in the shadow of those reads, and the common 4-bit output
//    has an epilogue of its own whose per-row constants were formed in the prologue.
//
// The four waves of a work-group are shared out over K parts (KS, partial sums added through
// LDS), pixel blocks side by side (NWT) and tile pairs (MS), KS*NWT*MS = 4: small grids split K,
// wide layers put the waves side by side, layers with many rows give every wave its own tile pair
// against the same patch.  The host picks the split per layer from a small cost model.
#pragma once
#include <hip/hip_runtime.h>

#include <utility>

#include "device_common.h"

namespace rmsmp {

constexpr int PW_THREADS = 256;
// bytes of leading scalar kernel arguments in front of the GemmArgs block (WIDE_FIRST_PARAMS below: twelve 4-byte slots)
constexpr int WIDE_FIRST_BYTES = 48;
static_assert(alignof(GemmArgs) <= 8, "the GemmArgs block must start right after the leading arguments");
constexpr int PW_PATCH_UNROLL = 6;  // 16-byte patch pieces in flight per thread, at most
// The patches of the 3x3 layers at hand are just under five pieces per thread (128 pixels plus halo
// x 8 pieces, 512 + halo x 2, ...), those of the 1x1 layers / GEMMs exactly six (64 x 24): a batch
// of five is one read, one decode and four registers less for the former.
constexpr int pw_batch(int taps) { return taps == 9 ? 5 : PW_PATCH_UNROLL; }
constexpr bool wide_has_gelu(int taps, int xb) { return taps == 1 && xb == 2; }
// Row metadata of a tile pair in LDS, field by field [field][64 rows]: rowscale bits, rowsum, original
// row, grouped position, and two values formed once per work-group for the lean 4-bit epilogue: the
// row's multiplier rowscale * activation scale (* 1/16 for shift-decoded tiles) and zero point * rowsum
// (* 16 for those tiles).
constexpr int PW_META_BYTES = 2 * TILE_M * 24;

struct WideGeom {
  int gx, gy;         // pixel tiles, row blocks (the launch grid is one-dimensional)
  int row_stride;     // LDS bytes per patch pixel (C + 16)
  int patch_rows;     // pixels staged per work-group
  int gather;         // 1: strided 1x1 layer, only the pixels that are used are staged (one per output pixel)
  int nchunk;         // 1x1 layers / GEMMs deeper than one LDS patch: the channels are staged nchunk parts of C, one after the other
  int pix_bytes;      // bytes of one input pixel in memory (all its channels)
  uint32_t magic_hw;  // ceil(2^32 / (OH*OW)), 0 when OH*OW == 1
  uint32_t magic_ow;  // ceil(2^32 / OW), 0 when OW == 1
};

// bytes of the partial-sum exchange buffer: every wave parks the blocks it does not finish
constexpr int pw_xch_bytes(int xb, int ks, int waves = 4) { return ks == 1 ? 0 : waves * (2 * xb - 2 * xb / ks) * 16 * LANES * 4; }

__device__ __forceinline__ int wide_fast_div(int n, uint32_t magic) {
  return magic ? (int)__umulhi((uint32_t)n, magic) : n;
}

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// Packed weight fragments are fetched through a buffer resource: the descriptor and the K-step
// offset live in scalar registers, the per-lane offset never changes, so stepping through K costs
// no vector instructions, and a read past the end of the tile returns zeros instead of faulting.
typedef unsigned v2w __attribute__((ext_vector_type(2)));
typedef unsigned v4w __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t wide_rsrc(const uint8_t* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}
template <int KIND>
__device__ __forceinline__ typename RawFrag<KIND>::type wide_load(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, int step_off) {
  if constexpr (KIND == TILE_I8) {
    const v4w w = __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, step_off, 0);
    return make_uint4(w.x, w.y, w.z, w.w);
  } else {
    const v2w w = __builtin_amdgcn_raw_buffer_load_b64(r, (int)lane_off, step_off, 0);
    return make_uint2(w.x, w.y);
  }
}

// Word CI (0..3) of a decoded weight fragment: the decode of a fragment is spread over the four
// pixel blocks of a K step, one word behind each pair of MFMAs.
template <int KIND, int CI>
__device__ __forceinline__ int decode_word(const typename RawFrag<KIND>::type& w, const uint4& T) {
  if constexpr (KIND == TILE_I8) {
    return (int)(CI == 0 ? w.x : CI == 1 ? w.y : CI == 2 ? w.z : w.w);
  } else {
    const uint32_t src = CI < 2 ? w.x : w.y;
    if constexpr (KIND == TILE_NIB_SHIFT) {
      return (int)((CI & 1) ? (src & 0xf0f0f0f0u) : ((src << 4) & 0xf0f0f0f0u));
    } else {
      return (int)lut4(((CI & 1) ? (src >> 4) : src) & 0x0f0f0f0fu, T);
    }
  }
}

// The first batch of patch reads is issued at the very start of the kernel, before the code of
// the work-group's class combination is even fetched; this is what it leaves behind.
struct WidePatchLoads {
  uint4 pw[PW_PATCH_UNROLL];
  __amdgpu_buffer_rsrc_t xr;  // the activation tensor
  uint32_t src0;              // byte offset of the patch in it
  int chunked, pix_bytes;     // chunked: a pixel's staged channels are only part of its pix_bytes bytes
  uint32_t x_last;            // last valid 16-byte read
  int f_lo;                   // first staged pixel
  // strided 1x1 layers (gather): piece idx belongs to output pixel n0 + idx / pieces-per-pixel
  int gather, n0, n_last, hw_out, OW, H, W, S;
  uint32_t magic_hw, magic_ow;
};

// 16-byte piece idx of the patch; reads past the end of X are clamped (those rows are never used)
template <int PIECES>
__device__ __forceinline__ uint4 wide_load_piece(const WidePatchLoads& pl, int idx) {
  uint32_t off = pl.src0 + (uint32_t)idx * 16u;
  if (pl.gather) {
    const int q = idx / PIECES, piece = idx - q * PIECES;
    int n = pl.n0 + q;
    n = n < pl.n_last ? n : pl.n_last;
    const int b = wide_fast_div(n, pl.magic_hw);
    const int rem = n - b * pl.hw_out;
    const int oh = wide_fast_div(rem, pl.magic_ow);
    const int ow = rem - oh * pl.OW;
    off = (uint32_t)((b * pl.H + oh * pl.S) * pl.W + ow * pl.S) * (uint32_t)(PIECES * 16) + (uint32_t)piece * 16u;
  }
  if (pl.chunked) {
    const int q = idx / PIECES, piece = idx - q * PIECES;
    off = pl.src0 + (uint32_t)q * (uint32_t)pl.pix_bytes + (uint32_t)piece * 16u;
  }
  off = off < pl.x_last ? off : pl.x_last;
  const v4w w = __builtin_amdgcn_raw_buffer_load_b128(pl.xr, (int)off, 0, 0);
  return make_uint4(w.x, w.y, w.z, w.w);
}

// Everything one wave does.  KIND0 / KIND1: storage classes of its two weight tiles.
template <int TAPS, int CPT, int XB, int KS, int NWT, int MS, bool DEEP, int KIND0, int KIND1>
__device__ __forceinline__ void wide_wave(const GemmArgs& a, const EpArgs& ea, const WideGeom& g, int bx, int pair,
                                          bool pair_live, WidePatchLoads& pl) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
  // waves per work-group: four in every split in use (eight, two per SIMD, measured no faster on
  // the benchmarked layer and is not instantiated)
  constexpr int NW = KS * NWT * MS;
  static_assert(NW == 4 || NW == 8, "four or eight waves");
  // The GELU epilogue (out_kind 3) exists where a transformer's feed-forward layer lands and the
  // register budget has room for it: plain GEMMs / 1x1 layers at 64 pixels per wave.  The host
  // sends such a layer nowhere else.
  constexpr bool WIDE_GELU = wide_has_gelu(TAPS, XB);
  constexpr int NT = LANES * NW;
  static_assert(XB == 2 || XB == 4, "32-pixel blocks per wave");
  constexpr int PW_XB = XB;
  constexpr int PW_WAVE_PX = 32 * XB;
  static_assert(CPT % KS == 0, "a tap must hold a whole number of K steps per wave");
  constexpr int C = CPT * KSTEP;
  constexpr int KW = TAPS == 9 ? 3 : 1;
  constexpr int KH = KW;
  constexpr int SPT = CPT / KS;       // K steps per tap and wave
  constexpr int NSTEP = TAPS * SPT;   // K steps per wave
  // loop body: one filter row while that stays small, else one tap
  constexpr int BT = (TAPS == 9 && SPT <= 4) ? 3 : 1;
  constexpr int BODY = BT * SPT;
  constexpr int NIT = TAPS / BT;
  // ring depth: a divisor of the body, so that a step's ring slot is the same in every iteration
  // (a ring of six steps measured no faster than four)
  constexpr int R = BODY % 4 == 0 ? 4 : BODY % 3 == 0 ? 3 : BODY % 2 == 0 ? 2 : 1;
  static_assert(R <= NSTEP, "ring deeper than the K loop");

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wt = wave % NWT;
  const int kq = wave / (NWT * MS);
  const int H = a.d.H, W = a.d.W, pad = a.d.pad, S = a.d.stride;
  const int hw_out = a.OH * a.OW;
  const int row_stride = g.row_stride, patch_rows = g.patch_rows;
  const int n0 = bx * (PW_WAVE_PX * NWT);  // first output pixel of the work-group
  const int nw = n0 + PW_WAVE_PX * wt;     // and of this wave

  // LDS: row metadata [MS pairs][4 fields][64 rows] | zero-point row (C bytes, +16 pad) | decoded
  // input patch.  The exchange buffer later lies over the zero-point row and the patch.
  uint8_t* const meta = smem_raw + PHASE_LDS_BYTES;
  uint8_t* const zrow = meta + MS * PW_META_BYTES;
  uint8_t* const patch = zrow + (C + 16);
  uint8_t* const xch = zrow;

  const int mt0 = pair, mt1 = a.w.n_tiles - 1 - pair;
  const TileRef tr0 = tile_ref(a.w, mt0), tr1 = tile_ref(a.w, mt1);
  const bool two = mt1 > mt0;

  // flattened input index of tap (0,0) for output pixel n (may be negative / out of image)
  // (pixel counts are below 2^23, checked by the host: the products are 24-bit multiplications,
  // which run at full rate where a 32-bit one takes four times as long)
  auto base_index = [&](int n, int& oh, int& ow) -> int {
    const int b = wide_fast_div(n, g.magic_hw);
    const int rem = n - __mul24(b, hw_out);
    oh = wide_fast_div(rem, g.magic_ow);
    ow = rem - __mul24(oh, a.OW);
    return __mul24(__mul24(b, H) + (__mul24(oh, S) - pad), W) + (__mul24(ow, S) - pad);
  };
  const int f_lo = pl.f_lo;

  // ---- weight stream of this wave: uniform base of its first K step + 32-bit lane offset
  constexpr int fb0 = KIND0 == TILE_I8 ? 16 : 8, fb1 = KIND1 == TILE_I8 ? 16 : 8;
  constexpr int step0 = LANES * fb0, step1 = LANES * fb1;  // bytes per K step
  // 1x1 layers deeper than one patch: the K loop runs once per part of the channels (see step 4)
  static_assert(!DEEP || TAPS == 1, "only 1x1 layers are staged in parts");
  const int nchunk = DEEP ? g.nchunk : 1;
  const int last_step = nchunk * NSTEP - 1;
  const __amdgpu_buffer_rsrc_t wb0 = wide_rsrc(a.w.blob + tr0.blob_off, (uint32_t)(nchunk * CPT * TAPS) * step0);
  const __amdgpu_buffer_rsrc_t wb1 = wide_rsrc(a.w.blob + tr1.blob_off, (uint32_t)(nchunk * CPT * TAPS) * step1);
  const uint32_t wl0 = (uint32_t)lane * fb0 + kq * step0, wl1 = (uint32_t)lane * fb1 + kq * step1;
  typename RawFrag<KIND0>::type ring0[R];
  typename RawFrag<KIND1>::type ring1[R];
  uint4 T0 = make_uint4(0, 0, 0, 0), T1 = T0;
  int4 meta_row = make_int4(0, 0, 0, 0);

  // ---- 1. the first batch of the patch is on its way; now what the wave's tile pair needs.
  // Pixels f_lo .. f_lo+patch_rows-1 are one contiguous byte range of X; piece idx (32 channels,
  // 16 bytes) sits at byte 16*idx of it and goes, decoded to int8, to LDS byte
  // 32*idx + 16*(idx / pieces-per-pixel) (rows are padded by 16 bytes).
  constexpr int PIECES = C / 32;
  const int total = patch_rows * PIECES;
  auto put_piece = [&](int idx, uint4 w) {
    uint8_t* dst = patch + idx * 32 + (idx / PIECES) * 16;
    *(v4i*)dst = decode_act_u4(make_uint2(w.x, w.y));
    *(v4i*)(dst + 16) = decode_act_u4(make_uint2(w.z, w.w));
  };
  uint4 (&pw)[PW_PATCH_UNROLL] = pl.pw;
  constexpr int PU = pw_batch(TAPS);
#pragma unroll
  for (int u = 0; u < R; ++u) {
    ring0[u] = wide_load<KIND0>(wb0, wl0, u * KS * step0);
    ring1[u] = wide_load<KIND1>(wb1, wl1, u * KS * step1);
  }
  if (KIND0 == TILE_NIB_LUT) T0 = *(const uint4*)(a.w.p_lut + ((int64_t)mt0 * TILE_M + tile_row_goff(lane & 31)) * 4);
  if (KIND1 == TILE_NIB_LUT) T1 = *(const uint4*)(a.w.p_lut + ((int64_t)mt1 * TILE_M + tile_row_goff(lane & 31)) * 4);
  // the wave with kq == 0 (and wt == 0) of a pair fetches its row metadata: lanes 0..31 tile 0, 32..63 tile 1
  if (kq == 0 && wt == 0) meta_row = ((const int4*)a.w.p_meta)[(lane < TILE_M ? mt0 : mt1) * TILE_M + (lane & (TILE_M - 1))];
  __builtin_amdgcn_sched_barrier(0);
  RMSMP_PHASE(11);

  // ---- 2. while those are in flight: accumulators, and per lane and 32-pixel block the LDS
  // address of tap (0,0), counted from the zero-point row, and the taps inside the image.
  // Validity is separable: tap (kh,kw) is inside iff kh is in [kh_lo,kh_hi] and kw in
  // [kw_lo,kw_hi].  A tap outside reads the zero-point row: its address is 0 whatever the lane, so
  // a tap's address is (address if inside) & (0 or -1).
  v16i acc[2][PW_XB];  // [weight tile][pixel block]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < PW_XB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
  const int lane_off = 16 * (lane >> 5) + kq * KSTEP;
  int dlt[PW_XB];
  uint32_t vm[PW_XB];
#pragma unroll
  for (int j = 0; j < PW_XB; ++j) {
    const int n = nw + 32 * j + (lane & 31);
    const bool n_ok = n < (int)a.N;
    int oh = 0, ow = 0;
    const int f0 = base_index(n_ok ? n : n0, oh, ow);
    const int kw_lo = max(0, pad - ow * S), kw_hi = min(KW - 1, W - 1 + pad - ow * S);
    const int kh_lo = max(0, pad - oh * S), kh_hi = min(KH - 1, H - 1 + pad - oh * S);
    const uint32_t wbits = kw_hi >= kw_lo ? ((2u << kw_hi) - (1u << kw_lo)) : 0u;  // bits kw_lo..kw_hi
    uint32_t m = 0;
#pragma unroll
    for (int kh = 0; kh < KH; ++kh) m |= (kh >= kh_lo && kh <= kh_hi) ? wbits << (KW * kh) : 0u;
    vm[j] = n_ok ? m : 0u;
    // (only 1x1 layers are ever gathered: the 3x3 kernels carry none of that code)
    dlt[j] = (C + 16) + __mul24((TAPS == 1 && g.gather) ? (n_ok ? n - n0 : 0) : f0 - f_lo, row_stride) + lane_off;
  }
  const int tap_row_bytes = W * row_stride;
  // LDS address (from zrow) of the lane's B fragments at tap t (wave-uniform; may be TAPS: nothing valid)
  auto tap_addr = [&](int t, int j) -> int {
    const int kh = KW == 1 ? 0 : (t * 11) >> 5;  // t / 3 for t <= 9
    const int kw = t - kh * KW;
    const int tapoff = kh * tap_row_bytes + kw * row_stride;
    return __builtin_amdgcn_sbfe((int)vm[j], t, 1) & (dlt[j] + tapoff);
  };
  // the zero-point row, for out-of-image taps
  {
    const uint32_t zf = 0x01010101u * (uint32_t)(a.ep.act_zero_point & 15);
    if (tid < C / 16) *(v4i*)(zrow + tid * 16) = (v4i){(int)zf, (int)zf, (int)zf, (int)zf};
  }
  __builtin_amdgcn_sched_barrier(0);
  RMSMP_PHASE(1);

  // ---- 3. the patch goes to LDS, batch by batch (the first batch is already in registers)
  auto stage_patch = [&](const int t0) {
#pragma unroll
    for (int u = 0; u < PU; ++u) {
      const int idx = u * NT + t0;
      if (idx < total) put_piece(idx, pw[u]);
    }
#pragma unroll 1
    for (int base = NT * PU; base < total; base += NT * PU) {
#pragma unroll
      for (int u = 0; u < PU; ++u) pw[u] = wide_load_piece<PIECES>(pl, base + u * NT + t0);
#pragma unroll
      for (int u = 0; u < PU; ++u) {
        const int idx = base + u * NT + t0;
        if (idx < total) put_piece(idx, pw[u]);
      }
    }
  };
  stage_patch(tid);
  // row metadata, field by field: [field][64 rows]
  if (kq == 0 && wt == 0) {
    const int ms = (wave / NWT) % MS;
    int* mf = (int*)(meta + ms * PW_META_BYTES) + lane;
    mf[0] = meta_row.x;
    mf[2 * TILE_M] = meta_row.y;
    mf[4 * TILE_M] = meta_row.z;
    mf[6 * TILE_M] = meta_row.w;
    const bool x16 = (lane < TILE_M ? KIND0 : KIND1) == TILE_NIB_SHIFT;
    mf[8 * TILE_M] = __float_as_int(__fmul_rn(__fmul_rn(__int_as_float(meta_row.x), ea.act_scale), x16 ? 0.0625f : 1.0f));
    mf[10 * TILE_M] = (x16 ? 16 * ea.zp : ea.zp) * meta_row.y;
  }
  // first weight fragments, and the refill of their ring slot
  v4i av0 = decode_raw<KIND0>(ring0[0], T0);
  v4i av1 = decode_raw<KIND1>(ring1[0], T1);
  if (R <= last_step) {
    ring0[0] = wide_load<KIND0>(wb0, wl0, R * KS * step0);
    ring1[0] = wide_load<KIND1>(wb1, wl1, R * KS * step1);
  }

  __syncthreads();  // patch, zero-point row and row metadata are in LDS

  RMSMP_PHASE(2);
  // ---- 4. K loop
#pragma unroll 1
  for (int ch = 0; ch < nchunk; ++ch) {
    // The next part of the channels replaces the patch: same pixels, pl.src0 moved on by C/2 bytes.
    // With 64 pixels per wave there are registers to spare, and the first batch of a part's reads
    // is issued before the previous part's K loop (PREFETCH); the piece addresses are formed again
    // for every part rather than kept in registers through the K loop.
    constexpr bool PREFETCH = DEEP && XB == 2;
    if (DEEP && ch > 0) {
      __syncthreads();  // every wave is done with the previous part
      int t0 = tid;
      asm volatile("" : "+v"(t0));
      if constexpr (!PREFETCH) {
        pl.src0 += C / 2;
#pragma unroll
        for (int u = 0; u < PU; ++u) pw[u] = wide_load_piece<PIECES>(pl, u * NT + t0);
      }
      stage_patch(t0);
      __syncthreads();
    }
    if (PREFETCH && ch + 1 < nchunk) {
      pl.src0 += C / 2;
      int t0 = tid;
      asm volatile("" : "+v"(t0));
#pragma unroll
      for (int u = 0; u < PU; ++u) pw[u] = wide_load_piece<PIECES>(pl, u * NT + t0);
    }
    const uint8_t* cur[PW_XB];  // LDS address of the lane's B fragment at the current tap
    v4i b[PW_XB];
#pragma unroll
    for (int j = 0; j < PW_XB; ++j) {
      cur[j] = zrow + tap_addr(0, j);
      b[j] = *(const v4i*)cur[j];
    }
    // Software pipeline, one K step = four sub-blocks, one per 32-pixel block j: the two MFMAs of
    // the block, then word j of both weight fragments of the NEXT step is decoded, then the
    // block's B fragment is re-read for the next step (its next use is six MFMAs away).  Nothing is
    // scheduled across sub-blocks, so every LDS read has that distance and the vector
    // instructions are spread evenly in the shadow of the matrix pipe.
    constexpr int NV0 = KIND0 == TILE_NIB_SHIFT ? 2 : KIND0 == TILE_NIB_LUT ? 6 : 0;
    constexpr int NV1 = KIND1 == TILE_NIB_SHIFT ? 2 : KIND1 == TILE_NIB_LUT ? 6 : 0;
    RMSMP_PHASE(14);
#pragma unroll 1
    for (int it = 0; it < NIT; ++it) {
#ifdef RMSMP_PHASE_TIMING
      if (it == 1) RMSMP_PHASE(7);
      if (it == 2) RMSMP_PHASE(10);
#endif
      static_for<0, BODY>([&](auto u_tag) {
        constexpr int u = decltype(u_tag)::value;
        constexpr bool wraps = u + 1 == BODY;
        constexpr int slot = (u + 1) % R;
        constexpr bool new_tap = (u + 1) % SPT == 0;
        constexpr int boff = ((u + 1) % SPT) * KS * KSTEP;
        constexpr int NVH = ((NV0 + NV1) * (4 / PW_XB) + (new_tap ? 3 : 0) + 1) / 2;  // vector instructions per MFMA slot
        // tap of the next step; with a filter row per iteration its row is the iteration number and
        // its column a constant, so that the tap's offset needs no division
        const int t = (it + (wraps ? 1 : 0)) * BT + (wraps ? 0 : (u + 1) / SPT);
        constexpr int kw_next = wraps ? 0 : (u + 1) / SPT;
        const int tapoff_next = BT == 3 ? (it + (wraps ? 1 : 0)) * tap_row_bytes + kw_next * row_stride : 0;
        v4i nav0, nav1;
        static_for<0, PW_XB>([&](auto j_tag) {
          constexpr int j = decltype(j_tag)::value;
          acc[0][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av0, b[j], acc[0][j], 0, 0, 0);
          acc[1][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av1, b[j], acc[1][j], 0, 0, 0);
          static_for<0, 4 / PW_XB>([&](auto c_tag) {
            constexpr int ci = j * (4 / PW_XB) + decltype(c_tag)::value;
            nav0[ci] = decode_word<KIND0, ci>(ring0[slot], T0);
            nav1[ci] = decode_word<KIND1, ci>(ring1[slot], T1);
          });
          if constexpr (new_tap) {
            if constexpr (BT == 3)
              cur[j] = zrow + (__builtin_amdgcn_sbfe((int)vm[j], t, 1) & (dlt[j] + tapoff_next));
            else
              cur[j] = zrow + tap_addr(t, j);
          }
          b[j] = *(const v4i*)(cur[j] + boff);
          if constexpr (j == PW_XB - 1) {
            // the ring slot is used up: refill it R steps further on
            int gs = ch * NSTEP + it * BODY + (u + 1 + R);
            gs = gs < last_step ? gs : last_step;  // past the end: any valid step
            ring0[slot] = wide_load<KIND0>(wb0, wl0, gs * (KS * step0));
            ring1[slot] = wide_load<KIND1>(wb1, wl1, gs * (KS * step1));
          }
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // MFMA
          __builtin_amdgcn_sched_group_barrier(0x002, NVH, 0);  // VALU
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // MFMA
          __builtin_amdgcn_sched_group_barrier(0x002, NVH, 0);  // VALU
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);    // the LDS read
          if constexpr (j == PW_XB - 1) __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);  // the ring loads
          __builtin_amdgcn_sched_barrier(0);
        });
        av0 = nav0;
        av1 = nav1;
#ifdef RMSMP_PHASE_TIMING
        if (u == 0 && it == 0) RMSMP_PHASE(15);
#endif
      });
    }
  }
  RMSMP_PHASE(3);

  // ---- 4. add the KS partial sums of a 64 x 128 block.  Its eight 32x32 blocks (weight tile t,
  // pixel block j: number 4t + j) are shared out among the KS waves: wave kq finishes blocks
  // kq*OWN .. kq*OWN+OWN-1 and parks the others in LDS for their owners.  The roles are KS copies
  // of the code under a wave-uniform branch, so that which accumulators are given and which are
  // kept is static.
  constexpr int NBLK = 2 * PW_XB;
  constexpr int OWN = NBLK / KS;
  v16i mine[OWN];
  if constexpr (KS == 1) {
#pragma unroll
    for (int q = 0; q < NBLK; ++q) mine[q] = acc[q / PW_XB][q % PW_XB];
  } else {
    __syncthreads();  // the exchange buffer overlays the patch: every wave is done reading it
    const int grp = wave % (NWT * MS);  // which 64 x 128 block of the work-group
    int* const blk = (int*)xch + grp * (KS * (NBLK - OWN) * 16 * LANES);
    // Which accumulators are given and which are kept depends on kq, and registers cannot be
    // indexed at run time: the two selections are KS copies of the code under a wave-uniform
    // branch.  The barrier and the reads of the others' blocks (addresses computed from kq) are
    // common code.  (With the barrier and the reads inside the per-role copies, hipcc 7.2 merged
    // the copies' tails and, in a variant with eight waves, left one role's first read address
    // unset: keep the roles free of barriers.)
    auto give = [&](auto kq_tag) {
      constexpr int KQ = decltype(kq_tag)::value;
      int* dst = blk + KQ * ((NBLK - OWN) * 16 * LANES);
      int gi = 0;
#pragma unroll
      for (int q = 0; q < NBLK; ++q) {
        if (q / OWN == KQ) continue;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          v4i gq;
#pragma unroll
          for (int e = 0; e < 4; ++e) gq[e] = acc[q / PW_XB][q % PW_XB][4 * c + e];
          *(v4i*)(dst + gi * (16 * LANES) + c * (4 * LANES) + lane * 4) = gq;
        }
        ++gi;
      }
#pragma unroll
      for (int o = 0; o < OWN; ++o) {
        constexpr int q0 = KQ * OWN;
        mine[o] = acc[(q0 + o) / PW_XB][(q0 + o) % PW_XB];
      }
    };
    if (kq == 0)
      give(std::integral_constant<int, 0>{});
    else if (kq == 1)
      give(std::integral_constant<int, 1>{});
    else if (KS == 4 && kq == 2)
      give(std::integral_constant<int, KS == 4 ? 2 : 0>{});
    else if (KS == 4)
      give(std::integral_constant<int, KS == 4 ? 3 : 0>{});
    __syncthreads();
    RMSMP_PHASE(4);
#pragma unroll
    for (int o = 0; o < OWN; ++o) {
      const int q = kq * OWN + o;
#pragma unroll
      for (int d = 1; d < KS; ++d) {
        // giver gk (every wave of the group but this one) put block q after the blocks before it
        // that are not its own: at position q if q comes before its own blocks, else OWN earlier
        const int gk = (kq + d) % KS;
        const int gi = q < gk * OWN ? q : q - OWN;
        const int* src = blk + gk * ((NBLK - OWN) * 16 * LANES) + gi * (16 * LANES);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const v4i got = *(const v4i*)(src + c * (4 * LANES) + lane * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) mine[o][4 * c + e] += got[e];
        }
      }
    }
  }
  RMSMP_PHASE(5);

  // ---- 5. epilogue: the blocks this wave finishes, tile by tile
  if (!pair_live) return;
  const int ms = (wave / NWT) % MS;
  const int* const meta_pair = (const int*)(meta + ms * PW_META_BYTES);
  constexpr int TPW = OWN >= PW_XB ? OWN / PW_XB : 1;  // weight tiles this wave finishes
  constexpr int BPT = OWN / TPW;                        // blocks per such tile
  constexpr int CH = BPT < 2 ? BPT : 2;                 // finished two at a time (register pressure)
  // The common case gets an epilogue of its own, chosen once per wave: 4-bit output, no bias, no
  // ReLU beyond the clamp at code 0 (a positive output scale makes the two the same), the whole
  // layer a multiple of 16 rows and the output 8-byte aligned.  Everything else goes through the
  // general finish_tiles.
  const bool lean = ea.out_kind == 2 && ea.bias == nullptr && !(ea.relu != 0 && !(ea.out_inv_scale > 0.0f)) &&
                    (ea.M & 15) == 0 && (((uintptr_t)ea.Y) & 7) == 0;
#pragma unroll
  for (int ti = 0; ti < TPW; ++ti) {
    const int q0 = kq * OWN + ti * BPT;  // first block
    const int my_tile = q0 / PW_XB;
    if (my_tile == 1 && !two) continue;
    RowMetaLds rm;
    rm.base = (const int*)__builtin_assume_aligned(meta_pair + my_tile * TILE_M + 16 * (lane >> 5), 64);
    rm.rows = 2 * TILE_M;
    const int n_rows = lane_rows(my_tile ? tr1.nvalid : tr0.nvalid, lane);
    const int kind = my_tile ? KIND1 : KIND0;
    const int64_t col0 = (int64_t)nw + 32 * (q0 % PW_XB) + (lane & 31);
    if (lean) {
      // 4-bit codes, no bias, no separate ReLU, all 16 rows of the lane alive: multipliers and
      // zero-point terms come ready from LDS, a pixel's 16 codes leave as one 8-byte store
      if (n_rows == 16) {
        float mrow[16], dummy[16];
        int crow[16];
        const float4* mp = (const float4*)(rm.base + 4 * (2 * TILE_M));
        const int4* cp = (const int4*)(rm.base + 5 * (2 * TILE_M));
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 mv = mp[q];
          mrow[4 * q] = mv.x, mrow[4 * q + 1] = mv.y, mrow[4 * q + 2] = mv.z, mrow[4 * q + 3] = mv.w;
        }
        if (ea.zp != 0) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int4 cv = cp[q];
            crow[4 * q] = cv.x, crow[4 * q + 1] = cv.y, crow[4 * q + 2] = cv.z, crow[4 * q + 3] = cv.w;
          }
        }
        RMSMP_GLOBAL uint8_t* const out0 = as_global((uint8_t*)ea.Y) + (rm.gpos0() >> 1);
#pragma unroll
        for (int o = 0; o < BPT; ++o) {
          v16i v = mine[ti * BPT + o];
          if (ea.zp != 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) v[r] -= crow[r];
          }
          uint32_t packed[2];
          requant_block<false, false>(v, mrow, dummy, ea.out_inv_scale, packed);
          const int64_t n = col0 + 32 * o;
          if (n < ea.N) *(RMSMP_GLOBAL v2u*)(out0 + n * (ea.M / 2)) = (v2u){packed[0], packed[1]};
        }
      }
      continue;
    }
    if constexpr (WIDE_GELU) {
      // the GELU epilogue holds twice the values per output: one block at a time, in a path of its own
      if (ea.out_kind == 3) {
#pragma unroll
        for (int o = 0; o < BPT; ++o) {
          const int64_t ncol[1] = {col0 + 32 * o};
          const v16i blocks[1] = {mine[ti * BPT + o]};
          finish_tiles<1, RowMetaLds, true, WIDE_FIRST_BYTES>(ea, kind, blocks, rm, n_rows, ncol);
        }
        continue;
      }
    }
#pragma unroll
    for (int c0 = 0; c0 < BPT; c0 += CH) {
      int64_t ncol[CH];
      v16i blocks[CH];
#pragma unroll
      for (int o = 0; o < CH; ++o) {
        ncol[o] = col0 + 32 * (c0 + o);
        blocks[o] = mine[ti * BPT + c0 + o];
      }
      finish_tiles<CH, RowMetaLds, false>(ea, kind, blocks, rm, n_rows, ncol);
    }
  }
  RMSMP_PHASE(6);
}

// block_id: the work-group's number within its layer (the launch's own work-group id, except in a
// launch that carries two layers)
// What a work-group needs before it can issue the reads of its input patch.  The kernels take
// these as leading scalar arguments (WIDE_FIRST_PARAMS), which the hardware hands over in
// registers at wave launch (kernel-argument preloading, -mllvm -amdgpu-kernarg-preload-count):
// the first read of the argument block from memory costs 450-700 cycles at the start of every
// launch, and nothing else can run before it.  The same values are in GemmArgs / WideGeom.
struct WideFirst {
  const void* X;
  int gx, gy;
  uint32_t magic_hw, magic_ow;
  int H, W, OH, OW, stride, pad, gather, B, pix_bytes;
  int64_t N;
};
#define WIDE_FIRST_PARAMS                                                                                         \
  const void *f_X, int f_gx, int f_gy, uint32_t f_magic_hw, uint32_t f_magic_ow, uint32_t f_hw, uint32_t f_ohw, \
      uint32_t f_spg, int f_B, int f_pix_bytes, int f_N
#define WIDE_FIRST_UNPACK()                                                                                   \
  WideFirst {                                                                                                 \
    f_X, f_gx, f_gy, f_magic_hw, f_magic_ow, (int)(f_hw & 0xffffu), (int)(f_hw >> 16), (int)(f_ohw & 0xffffu), \
        (int)(f_ohw >> 16), (int)(f_spg & 0xffu), (int)((f_spg >> 8) & 0xffu), (int)(f_spg >> 16), f_B,       \
        f_pix_bytes, (int64_t)f_N                                                                             \
  }
__device__ __forceinline__ WideFirst wide_first_of(const GemmArgs& a, const WideGeom& g) {
  return WideFirst{a.X, g.gx, g.gy, g.magic_hw, g.magic_ow, a.d.H, a.d.W, a.OH, a.OW, a.d.stride, a.d.pad, g.gather, a.d.B, g.pix_bytes, a.N};
}

template <int TAPS, int CPT, int XB, int KS, int NWT, int MS, bool DEEP>
__device__ __forceinline__ void wide_kernel_impl(const WideFirst& f, const GemmArgs& a, const WideGeom& g, const unsigned block_id) {
  RMSMP_PHASE(0);
  // Work-group id -> (pixel tile bx, row block by).  Consecutive ids go to different XCDs, each
  // with its own L2, so the gy work-groups that read the same input patch get ids that are equal
  // modulo 8 and follow each other on that XCD: the patch comes out of memory once, not gy
  // times.  The grid is padded to a multiple of 8 pixel tiles; the extra work-groups leave.
  const int xcd = block_id & 7, slot = block_id >> 3;
  const int by = slot % f.gy;
  const int bx = (slot / f.gy) * 8 + xcd;
  if (bx >= f.gx) return;
  // first of all, the reads of the input patch: they depend on nothing but the pixel tile
  WidePatchLoads pl;
  {
    const int n0 = bx * (32 * XB * NWT);
    const int hw_out = f.OH * f.OW;
    const int b = wide_fast_div(n0, f.magic_hw);
    const int rem = n0 - b * hw_out;
    const int oh = wide_fast_div(rem, f.magic_ow);
    const int ow = rem - oh * f.OW;
    int f_lo = (b * f.H + (oh * f.stride - f.pad)) * f.W + (ow * f.stride - f.pad);
    f_lo = f_lo < 0 ? 0 : f_lo;
    const uint32_t x_bytes = (uint32_t)(f.B * f.H * f.W) * (uint32_t)f.pix_bytes;
    pl.f_lo = f_lo;
    pl.xr = wide_rsrc((const uint8_t*)f.X, x_bytes);
    pl.src0 = (uint32_t)f_lo * (uint32_t)f.pix_bytes;
    pl.chunked = DEEP, pl.pix_bytes = f.pix_bytes;
    pl.x_last = x_bytes - 16u;
    pl.gather = TAPS == 1 ? f.gather : 0, pl.n0 = n0, pl.n_last = (int)f.N - 1, pl.hw_out = hw_out, pl.OW = f.OW;
    pl.H = f.H, pl.W = f.W, pl.S = f.stride, pl.magic_hw = f.magic_hw, pl.magic_ow = f.magic_ow;
    if (TAPS == 1 && f.gather) pl.f_lo = 0;
#pragma unroll
    for (int u = 0; u < pw_batch(TAPS); ++u) pl.pw[u] = wide_load_piece<CPT>(pl, u * (LANES * KS * NWT * MS) + (int)threadIdx.x);
  }
  EpArgs ea = pin_epilogue_args(a);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n_pairs = (a.w.n_tiles + 1) / 2;
  // Pair y is tile y and tile n_tiles-1-y: tiles are sorted by class, so a table-decoded tile is
  // paired with a cheap one whenever the layer has both.  A wave past the last pair repeats it
  // (it takes part in every barrier) and stores nothing.
  int pair = by * MS + (wave / NWT) % MS;
  const bool pair_live = pair < n_pairs;
  pair = pair_live ? pair : n_pairs - 1;
  auto kind_of = [&](int mt) { return mt < a.w.class_tiles[0] ? 0 : mt < a.w.class_tiles[0] + a.w.class_tiles[1] ? 1 : 2; };
  const int k0 = kind_of(pair), k1 = kind_of(a.w.n_tiles - 1 - pair);
#define RMSMP_WIDE(K0, K1) \
  if (k0 == K0 && k1 == K1) wide_wave<TAPS, CPT, XB, KS, NWT, MS, DEEP, K0, K1>(a, ea, g, bx, pair, pair_live, pl);
  RMSMP_WIDE(TILE_NIB_SHIFT, TILE_NIB_SHIFT)
  else RMSMP_WIDE(TILE_NIB_SHIFT, TILE_NIB_LUT)
  else RMSMP_WIDE(TILE_NIB_SHIFT, TILE_I8)
  else RMSMP_WIDE(TILE_NIB_LUT, TILE_NIB_LUT)
  else RMSMP_WIDE(TILE_NIB_LUT, TILE_I8)
  else RMSMP_WIDE(TILE_I8, TILE_I8)
#undef RMSMP_WIDE
  RMSMP_PHASE_FLUSH();
}

template <int TAPS, int CPT, int XB, int KS, int NWT, int MS, bool DEEP>
__global__ __launch_bounds__(LANES * KS * NWT * MS, KS * NWT * MS == 8 ? 1 : 2) void conv_wide_kernel(WIDE_FIRST_PARAMS, GemmArgs a, WideGeom g) {
  wide_kernel_impl<TAPS, CPT, XB, KS, NWT, MS, DEEP>(WIDE_FIRST_UNPACK(), a, g, blockIdx.x);
}

// Two layers that read the same input tensor as one launch: a 3x3 layer and a 1x1 layer with the
// same channel count (the two convolutions at the head of a residual stage, Section 4.2's
// ResNet-18: the stride-2 3x3 convolution and the stride-2 1x1 projection of the shortcut).  The
// first blocks_a work-groups run the 3x3 layer's code, the others the 1x1 layer's; the two kinds
// share compute units, so the short 1x1 work-groups run in the shadow of the long ones instead
// of paying a launch of their own.  Neither layer may use the GELU epilogue (its table is read
// from the start of the kernel arguments).
struct WidePairSplit {
  int xa, ka, na, ma;  // 3x3 layer: pixel blocks per wave, K split, side by side, tile pairs
  int xb, kb, nb, mb;  // 1x1 layer
};
// the splits the pair kernel is built with, per channel count / 32: those the single-layer model
// picks for the ResNet-18 stage heads at batch 64
constexpr WidePairSplit wide_pair_split(int cpt) {
  return cpt == 2 ? WidePairSplit{4, 2, 1, 2, 2, 1, 4, 1} : cpt == 4 ? WidePairSplit{2, 1, 1, 4, 2, 1, 1, 4} : WidePairSplit{2, 2, 1, 2, 2, 2, 1, 2};
}

template <int CPT>
__global__ __launch_bounds__(LANES * 4, 2) void conv_wide_pair_kernel(WIDE_FIRST_PARAMS, GemmArgs a, WideGeom ga, GemmArgs b, WideGeom gb, unsigned blocks_a) {
  // (the leading arguments are the 3x3 layer's; the 1x1 layer's work-groups read theirs from memory)
  constexpr WidePairSplit sp = wide_pair_split(CPT);
  if (blockIdx.x < blocks_a)
    wide_kernel_impl<9, CPT, sp.xa, sp.ka, sp.na, sp.ma, false>(WIDE_FIRST_UNPACK(), a, ga, blockIdx.x);
  else
    wide_kernel_impl<1, CPT, sp.xb, sp.kb, sp.nb, sp.mb, false>(wide_first_of(b, gb), b, gb, blockIdx.x - blocks_a);
}

struct WidePlan {
  GemmArgs a;  // the argument block (a plain GEMM becomes a 1x1 convolution over N single-pixel images)
  WideGeom g;
  size_t lds = 0;
  unsigned blocks = 0;
  int xb = 4, ks = 1, nwt = 1, ms = 1;
  int cpt = 0;  // K steps of 32 channels staged at a time (the kernel family)
};

// the leading scalar arguments of a launch, from its plan (sizes are checked by the host: image
// sides below 2^16, stride and padding below 2^8, pixel counts below 2^23)
#define WIDE_FIRST_ARGS(p)                                                                                              \
  (p).a.X, (p).g.gx, (p).g.gy, (p).g.magic_hw, (p).g.magic_ow, (uint32_t)(p).a.d.H | ((uint32_t)(p).a.d.W << 16),        \
      (uint32_t)(p).a.OH | ((uint32_t)(p).a.OW << 16),                                                                  \
      (uint32_t)(p).a.d.stride | ((uint32_t)(p).a.d.pad << 8) | ((uint32_t)(p).g.gather << 16), (int)(p).a.d.B,        \
      (p).g.pix_bytes, (int)(p).a.N

template <int TAPS, int CPT, int XB, int KS, int NWT, int MS, bool DEEP>
inline int launch_wide_t(const WidePlan& p, hipStream_t s) {
  if constexpr (CPT % KS != 0 || TAPS * (CPT / KS) < 2) {
    return (int)hipErrorInvalidValue;
  } else {
    static std::atomic<uint64_t> allowed{0};
    if (const int rc = allow_large_lds((const void*)conv_wide_kernel<TAPS, CPT, XB, KS, NWT, MS, DEEP>, allowed)) return rc;
    hipLaunchKernelGGL((conv_wide_kernel<TAPS, CPT, XB, KS, NWT, MS, DEEP>), dim3(p.blocks), dim3(LANES * KS * NWT * MS), p.lds, s, WIDE_FIRST_ARGS(p), p.a, p.g);
    return (int)hipGetLastError();
  }
}

template <int CPT>
inline int launch_wide_pair_t(const WidePlan& pa, const WidePlan& pb, hipStream_t s) {
  static std::atomic<uint64_t> allowed{0};
  if (const int rc = allow_large_lds((const void*)conv_wide_pair_kernel<CPT>, allowed)) return rc;
  const size_t lds = pa.lds > pb.lds ? pa.lds : pb.lds;
  hipLaunchKernelGGL((conv_wide_pair_kernel<CPT>), dim3(pa.blocks + pb.blocks), dim3(LANES * 4), lds, s, WIDE_FIRST_ARGS(pa), pa.a, pa.g, pb.a, pb.g, pa.blocks);
  return (int)hipGetLastError();
}

template <int TAPS, int CPT, bool DEEP>
inline int launch_wide_tc(const WidePlan& p, hipStream_t s) {
  if (p.xb == 4 && p.ks == 4 && p.nwt == 1 && p.ms == 1) return launch_wide_t<TAPS, CPT, 4, 4, 1, 1, DEEP>(p, s);
  if (p.xb == 4 && p.ks == 2 && p.nwt == 2 && p.ms == 1) return launch_wide_t<TAPS, CPT, 4, 2, 2, 1, DEEP>(p, s);
  if (p.xb == 4 && p.ks == 1 && p.nwt == 4 && p.ms == 1) return launch_wide_t<TAPS, CPT, 4, 1, 4, 1, DEEP>(p, s);
  if (p.xb == 4 && p.ks == 1 && p.nwt == 1 && p.ms == 4) return launch_wide_t<TAPS, CPT, 4, 1, 1, 4, DEEP>(p, s);
  if (p.xb == 2 && p.ks == 2 && p.nwt == 2 && p.ms == 1) return launch_wide_t<TAPS, CPT, 2, 2, 2, 1, DEEP>(p, s);
  if (p.xb == 2 && p.ks == 4 && p.nwt == 1 && p.ms == 1) return launch_wide_t<TAPS, CPT, 2, 4, 1, 1, DEEP>(p, s);
  if (p.xb == 2 && p.ks == 1 && p.nwt == 1 && p.ms == 4) return launch_wide_t<TAPS, CPT, 2, 1, 1, 4, DEEP>(p, s);
  if (p.xb == 2 && p.ks == 1 && p.nwt == 4 && p.ms == 1) return launch_wide_t<TAPS, CPT, 2, 1, 4, 1, DEEP>(p, s);
  if (p.xb == 4 && p.ks == 2 && p.nwt == 1 && p.ms == 2) return launch_wide_t<TAPS, CPT, 4, 2, 1, 2, DEEP>(p, s);
  if (p.xb == 2 && p.ks == 2 && p.nwt == 1 && p.ms == 2) return launch_wide_t<TAPS, CPT, 2, 2, 1, 2, DEEP>(p, s);
  return (int)hipErrorInvalidValue;
}


}  // namespace rmsmp
