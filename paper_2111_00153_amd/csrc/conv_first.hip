// First-layer convolution kernel of librmsmp (gfx950): three input channels, 8-bit activations,
// square filter of 3, 5 or 7 taps a side, stride 2, odd padding (the 7x7 / stride-2 / pad-3 first
// layer of the ResNets of Section 4, which the paper keeps at 8 bits).
//
// The lowered matrix of such a layer is ~50x its input and its output is the largest tensor of
// the network, so the kernel is bound by the epilogue's vector instructions and by memory, not by
// the matrix cores.  What it does about that:
//  * Nothing is lowered.  Weights are stored one K step per filter row (element (kh, kw, c) at
//    kh*32 + kw*4 + c), so a lane's B fragment for filter row kh is four consecutive input pixels
//    (padded to four bytes each) of input row 2*oh - pad + kh.
//  * A work-group walks through several 16x16 tiles of output pixels; each wave holds the weights
//    of one weight tile in registers the whole time and takes half of the rows of every pixel
//    tile (the narrower kernel fetched the weights again for every 128 pixels: 14 KiB per wave
//    against 0.4 KiB of input).  Three work-groups share a compute unit; the launch has exactly
//    768 of them when there are that many tiles, with the tiles spread evenly, so every compute
//    unit carries the same load in a single round.
//  * The input pixels of a tile are staged in LDS already in MFMA operand order: the staging
//    thread reads 16 aligned bytes (four pixels), and seven vector instructions turn them into the
//    16 bytes two fragments will read, so the inner loop has no byte shuffles at all.  Tiles whose
//    staged columns lie inside the image skip the padding masks.
//  * The next tile's input is fetched while the current tile is multiplied, and written to the
//    other LDS buffer afterwards: one barrier per tile.  A pass issues all its loads (first tile,
//    packed weights, row metadata) before it waits for any of them.
//  * The kernel is bound by vector instructions (a wave's vector instruction costs 4 to 5 cycles
//    of its SIMD, and the 4-bit epilogue needs five per output value: convert, two roundings of
//    the scale product, clamp, pack), so the common case has a loop of its own (template
//    parameter chosen by the host) that carries nothing else: row multipliers in registers, the
//    four blocks of a tile in one piece of straight-line code, 4-bit codes stored through a
//    buffer descriptor whose per-lane offset is fixed for the pass.
#include <hip/hip_runtime.h>

#include "device_common.h"

namespace rmsmp {

constexpr int CF_T = 16;         // output tile: 16 x 16 pixels
constexpr int CF_UNITS = 10;     // staged 16-byte units (four pixels each) per input row
constexpr int CF_ROWB = CF_UNITS * 16;
constexpr int CF_MAX_TILES = 64;  // row metadata of all weight tiles sits in LDS (512 bytes per tile)

struct FirstGeom {
  int tiles_w, tiles_h;   // 16x16 output tiles per image
  int total_tiles;        // B * tiles_h * tiles_w
  int tiles_base, tiles_rem;  // work-group i takes tiles_base tiles, one more when i < tiles_rem
  uint32_t magic_tw;      // ceil(2^32 / tiles_w), 0 when tiles_w == 1
  uint32_t magic_thw;     // ceil(2^32 / (tiles_w * tiles_h)), 0 when that is 1
};

__device__ __forceinline__ int cf_fast_div(int n, uint32_t magic) {
  return magic ? (int)__umulhi((uint32_t)n, magic) : n;
}

typedef unsigned cf_v4w __attribute__((ext_vector_type(4)));

template <int KHW, int MODE_>
__global__ __launch_bounds__(256, 3) void conv_first_kernel(GemmArgs a, FirstGeom g) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
  constexpr int PH = 2 * (CF_T - 1) + KHW;   // staged input rows per tile
  constexpr int BUF = PH * CF_ROWB;          // bytes per staging buffer
  constexpr int NUNIT = PH * CF_UNITS;
  constexpr int UPT = (NUNIT + 255) / 256;   // units per thread
  const EpArgs ea = pin_epilogue_args(a);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int H = a.d.H, W = a.d.W, pad = a.d.pad;
  uint8_t* const buf0 = smem_raw;
  int* const meta = (int*)(smem_raw + 2 * BUF);  // [tile][field][32 rows]
  // per padded row: multiplier rowscale * act_scale (* 1/16 for shift-decoded tiles) and bias
  float* const mtab = (float*)(meta + a.w.n_tiles * (4 * TILE_M));
  float* const btab = mtab + a.w.n_tiles * TILE_M;

  const int wg = blockIdx.x;
  const int t_lo = wg * g.tiles_base + min(wg, g.tiles_rem);
  const int t_hi = t_lo + g.tiles_base + (wg < g.tiles_rem ? 1 : 0);
  if (t_lo >= t_hi) return;

  const uint32_t x_bytes = (uint32_t)(a.d.B * H * W) * 3u;
  const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc((void*)a.X, 0, (int)x_bytes, 0x00020000);
  const uint32_t z = (uint32_t)a.ep.act_zero_point & 255u;
  const uint32_t zA = z * 0x01010101u, zB = z * 0x00010001u;  // (c0,c2,c0,c2) and (c1,-,c1,-) of two padding pixels

  // tile id -> image, first output row / column, first staged input row / pixel
  struct TilePos {
    int b, oh0, ow0, ih0, iw_s, shift;
  };
  auto tile_pos = [&](int t) -> TilePos {
    TilePos p;
    p.b = cf_fast_div(t, g.magic_thw);
    const int r = t - p.b * (g.tiles_w * g.tiles_h);
    const int th = cf_fast_div(r, g.magic_tw);
    const int tw = r - th * g.tiles_w;
    p.oh0 = th * CF_T;
    p.ow0 = tw * CF_T;
    p.ih0 = p.oh0 * 2 - pad;
    // pixel pairs are staged from an odd pixel on; the first staged pixel iw_s + 1 is the last odd
    // position at or before the first pixel needed (2*ow0 - pad, pad odd) with iw_s a multiple of 4
    const int first = p.ow0 * 2 - pad - 1;       // even
    p.iw_s = first & ~3;                          // (also right for negative values)
    p.shift = (first - p.iw_s) >> 1;              // 0 or 1: pair index of the first pixel needed
    return p;
  };

  // ---- staging: unit (r, u) of a tile = pixels iw_s+1+4u .. iw_s+4+4u of input row ih0 + r
  auto unit_offset = [&](const TilePos& p, int id, bool& row_ok) -> uint32_t {
    const int r = id / CF_UNITS, u = id - r * CF_UNITS;
    const int ih = p.ih0 + r;
    row_ok = id < NUNIT && ih >= 0 && ih < H;
    // 16 aligned bytes holding the unit's 12 at bytes 3..14; -12 for the first unit of the tensor's
    // very first row when iw_s = -4 (see fetch_units)
    return (uint32_t)(((p.b * H + ih) * W + p.iw_s) * 3 + 12 * u);
  };
  auto fetch_units = [&](const TilePos& p, cf_v4w (&raw)[UPT]) {
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
      bool row_ok;
      const uint32_t off = unit_offset(p, tid + 256 * i, row_ok);
      raw[i] = (cf_v4w){0u, 0u, 0u, 0u};
      // Only offset -12 can be negative (iw_s >= -4): three of the unit's pixels lie left of the
      // image and the fourth is the tensor's first pixel.  Read from 0 and move it to its place.
      const bool before = (int)off < 0;
      if (row_ok) raw[i] = __builtin_amdgcn_raw_buffer_load_b128(xr, before ? 0 : (int)off, 0, 0);
      if (before) raw[i].w = raw[i].x;
    }
  };
  auto store_units = [&](const TilePos& p, const cf_v4w (&raw)[UPT], uint8_t* buf) {
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
      const int id = tid + 256 * i;
      if (id >= NUNIT) continue;
      const int r = id / CF_UNITS, u = id - r * CF_UNITS;
      const int ih = p.ih0 + r;
      const bool row_ok = ih >= 0 && ih < H;
      const int iw = p.iw_s + 1 + 4 * u;  // first of the unit's four pixels
      // bytes 3..14 of the 16 read: pixels a, b, c, d, three channels each
      const uint32_t e = __builtin_amdgcn_alignbyte(raw[i].y, raw[i].x, 3);  // a0 a1 a2 b0
      const uint32_t f = __builtin_amdgcn_alignbyte(raw[i].z, raw[i].y, 3);  // b1 b2 c0 c1
      const uint32_t h = __builtin_amdgcn_alignbyte(raw[i].w, raw[i].z, 3);  // c2 d0 d1 d2
      // operand words of the pixel pairs (a,b) and (c,d): even channels, odd channels (channel 3 = 0)
      uint32_t A0 = __builtin_amdgcn_perm(f, e, 0x05030200u);  // a0 a2 b0 b2
      uint32_t B0 = __builtin_amdgcn_perm(f, e, 0x0c040c01u);  // a1 0  b1 0
      uint32_t A1 = __builtin_amdgcn_perm(h, f, 0x07050402u);  // c0 c2 d0 d2
      uint32_t B1 = __builtin_amdgcn_perm(h, f, 0x0c060c03u);  // c1 0  d1 0
      // a tile whose staged columns all lie inside the image, with zero point 0: nothing to mask
      // (rows outside the image were fetched as zeros)
      if (z == 0 && p.iw_s + 1 >= 0 && p.iw_s + 1 + 4 * CF_UNITS <= W) {
        *(v4i*)(buf + r * CF_ROWB + u * 16) = (v4i){(int)A0, (int)B0, (int)A1, (int)B1};
        continue;
      }
      // pixels outside the image hold the zero point
      const uint32_t va = (row_ok && iw >= 0 && iw < W) ? 0x0000ffffu : 0u;
      const uint32_t vb = (row_ok && iw + 1 >= 0 && iw + 1 < W) ? 0xffff0000u : 0u;
      const uint32_t vc = (row_ok && iw + 2 >= 0 && iw + 2 < W) ? 0x0000ffffu : 0u;
      const uint32_t vd = (row_ok && iw + 3 >= 0 && iw + 3 < W) ? 0xffff0000u : 0u;
      const uint32_t m0 = va | vb, m1 = vc | vd;
      A0 = (A0 & m0) | (zA & ~m0);
      B0 = (B0 & m0) | (zB & ~m0);
      A1 = (A1 & m1) | (zA & ~m1);
      B1 = (B1 & m1) | (zB & ~m1);
      *(v4i*)(buf + r * CF_ROWB + u * 16) = (v4i){(int)A0, (int)B0, (int)A1, (int)B1};
    }
  };

  // ---- row metadata of every weight tile, field by field
  auto stage_metadata = [&]() {
  for (int idx = tid; idx < a.w.n_tiles * TILE_M; idx += 256) {
    const int4 m = ((const int4*)a.w.p_meta)[idx];
    int* dst = meta + (idx / TILE_M) * (4 * TILE_M) + (idx % TILE_M);
    dst[0] = m.x;
    dst[TILE_M] = m.y;
    dst[2 * TILE_M] = m.z;
    dst[3 * TILE_M] = m.w;
    const float fold = tile_ref(a.w, idx / TILE_M).kind == TILE_NIB_SHIFT ? 0.0625f : 1.0f;
    mtab[idx] = __fmul_rn(__fmul_rn(__int_as_float(m.x), ea.act_scale), fold);
    btab[idx] = ea.bias ? as_global(ea.bias)[m.z < 0 ? 0 : m.z] : 0.0f;
  }
  };

  // this lane's output pixel inside a 2-row x 16-column block, and its fragment offset in a staged row
  const int pr = (lane & 31) >> 4, pc = lane & 15, hh = lane >> 5;

  // ---- weight tiles two at a time; all pixel tiles of the work-group against them.  A wave
  // holds the weights of ONE tile (even waves the first of the two, odd waves the second) and
  // takes half of a pixel tile's rows: few registers per wave, so that four work-groups share a
  // compute unit and hide each other's LDS, MFMA and store latencies.
  const TilePos pos0 = tile_pos(t_lo);
#pragma unroll 1
  for (int mt0 = 0; mt0 < a.w.n_tiles; mt0 += 2) {
    const bool mine_live = mt0 + (wave & 1) < a.w.n_tiles;
    const int mt = mine_live ? mt0 + (wave & 1) : mt0;
    const TileRef tr = tile_ref(a.w, mt);
    // All loads of the pass are issued before anything waits: the first pixel tile, the packed
    // weight fragments of the KHW filter rows and (first pass) the row metadata.
    cf_v4w raw0[UPT];
    fetch_units(pos0, raw0);
    uint4 wr[KHW];
    uint4 T = make_uint4(0, 0, 0, 0);
    {
      const uint8_t* wp = a.w.blob + tr.blob_off;
      if (tr.kind == TILE_I8) {
#pragma unroll
        for (int kh = 0; kh < KHW; ++kh) wr[kh] = load_raw<TILE_I8>(wp, (uint32_t)(kh * LANES + lane) * 16);
      } else {
#pragma unroll
        for (int kh = 0; kh < KHW; ++kh) {
          const uint2 v = load_raw<TILE_NIB_SHIFT>(wp, (uint32_t)(kh * LANES + lane) * 8);
          wr[kh] = make_uint4(v.x, v.y, 0, 0);
        }
        if (tr.kind == TILE_NIB_LUT) T = *(const uint4*)(a.w.p_lut + ((int64_t)mt * TILE_M + tile_row_goff(lane & 31)) * 4);
      }
    }
    if (mt0 == 0) stage_metadata();
    // decoded weight fragments, kept for all pixel tiles
    v4i av[KHW];
    if (tr.kind == TILE_I8) {
#pragma unroll
      for (int kh = 0; kh < KHW; ++kh) av[kh] = decode_raw<TILE_I8>(wr[kh], T);
    } else if (tr.kind == TILE_NIB_SHIFT) {
#pragma unroll
      for (int kh = 0; kh < KHW; ++kh) av[kh] = decode_raw<TILE_NIB_SHIFT>(make_uint2(wr[kh].x, wr[kh].y), T);
    } else {
#pragma unroll
      for (int kh = 0; kh < KHW; ++kh) av[kh] = decode_raw<TILE_NIB_LUT>(make_uint2(wr[kh].x, wr[kh].y), T);
    }
    // (decoded once: the fragments stay in registers, not re-derived from the packed words per tile)
#pragma unroll
    for (int kh = 0; kh < KHW; ++kh) asm volatile("" : "+v"(av[kh]));
    TilePos pos = pos0;
    __syncthreads();  // metadata stored / previous pass done with both buffers
    store_units(pos0, raw0, buf0);
    __syncthreads();

    const int n_rows = mine_live ? lane_rows(tr.nvalid, lane) : 0;
    const int gpos0 = meta[mt * (4 * TILE_M) + 16 * hh + 3 * TILE_M];
    // a lane's 16 codes of a pixel leave as one 8-byte store when all 16 rows exist and the place is aligned
    const int64_t row_bytes = ea.M / 2;
    const bool whole = n_rows == 16 && (row_bytes & 7) == 0 && ((((uintptr_t)ea.Y) + (gpos0 >> 1)) & 7) == 0;
    // 4-bit output as a buffer (only used when it is below 2 GiB, see the choice of the loop below)
    const __amdgpu_buffer_rsrc_t yr = __builtin_amdgcn_make_buffer_rsrc((void*)ea.Y, 0, (int)(ea.N * row_bytes), 0x00020000);
    const int s_row = a.OW * (int)row_bytes;
    const int lane_off = (pr * a.OW + pc) * (int)row_bytes + (gpos0 >> 1);

    // The pixel-tile loop exists three times (kernel template parameter, chosen by the host), so that the common
    // 4-bit-output case carries neither the other output kinds nor the optional steps:
    // MODE 1: 4-bit output, zero point 0, no bias, no separate ReLU (with a positive output scale the
    //         clamp at code 0 does what ReLU would); MODE 2: 4-bit output, zero point 0, anything
    //         else; MODE 0: every other epilogue, through the general finish_tiles.
    // the lean loop keeps its 16 row multipliers in registers
    float mkeep[16];
    {
      const float4* mp = (const float4*)(mtab + mt * TILE_M + 16 * hh);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 mv = mp[q];
        mkeep[4 * q] = mv.x, mkeep[4 * q + 1] = mv.y, mkeep[4 * q + 2] = mv.z, mkeep[4 * q + 3] = mv.w;
      }
    }
    auto run_tiles = [&](auto mode_tag) {
      constexpr int MODE = decltype(mode_tag)::value;
#pragma unroll 1
      for (int t = t_lo; t < t_hi; ++t) {
        const int cur = (t - t_lo) & 1;
        const uint8_t* buf = buf0 + cur * BUF;
        const bool more = t + 1 < t_hi;
        TilePos nxt = pos;
        cf_v4w raw[UPT];
        if (more) {
          nxt = tile_pos(t + 1);
          fetch_units(nxt, raw);
        }
        const int s_tile = ((pos.b * a.OH + pos.oh0) * a.OW + pos.ow0) * (int)row_bytes;  // (used by 4-bit stores only)
        const bool col_ok = pos.ow0 + pc < a.OW;
        // ---- this wave's four blocks (rows 8*(w/2) .. 8*(w/2)+7 of the tile) against its weight tile
        auto do_block = [&](const int bl) {
          const int oh_l = 8 * (wave >> 1) + 2 * bl + pr;
          const uint8_t* fp = buf + (oh_l * 2) * CF_ROWB + (pc + 2 * hh + pos.shift) * 8;
          v4i bf[KHW];
#pragma unroll
          for (int kh = 0; kh < KHW; ++kh) {
            const uint2 lo = *(const uint2*)(fp + kh * CF_ROWB);
            const uint2 hi = *(const uint2*)(fp + kh * CF_ROWB + 8);
            bf[kh] = (v4i){(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
          }
          v16i acc[1];
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[0][r] = 0;
#pragma unroll
          for (int kh = 0; kh < KHW; ++kh) acc[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av[kh], bf[kh], acc[0], 0, 0, 0);
          const int oh = pos.oh0 + oh_l, ow = pos.ow0 + pc;
          const bool px_ok = oh < a.OH && ow < a.OW;
          const int64_t n = px_ok ? ((int64_t)pos.b * a.OH + oh) * a.OW + ow : a.N;  // a.N = no store
          if constexpr (MODE == 0) {
            RowMetaLds rm;
            rm.base = (const int*)__builtin_assume_aligned(meta + mt * (4 * TILE_M) + 16 * hh, 64);
            rm.rows = TILE_M;
            const int64_t ncol[1] = {n};
            finish_tiles<1, RowMetaLds, false>(ea, tr.kind, acc, rm, n_rows, ncol);  // (no GELU epilogue here)
          } else {
            uint32_t packed[2];
            float brow[16];
            const int row0 = mt * TILE_M + 16 * hh;
            if constexpr (MODE == 1) {
              requant_block<false, false>(acc[0], mkeep, brow, ea.out_inv_scale, packed);
            } else {
              float mrow[16];
              const float4* mp = (const float4*)(mtab + row0);
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const float4 mv = mp[q];
                mrow[4 * q] = mv.x, mrow[4 * q + 1] = mv.y, mrow[4 * q + 2] = mv.z, mrow[4 * q + 3] = mv.w;
              }
              const float4* bp = (const float4*)(btab + row0);
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const float4 bv = bp[q];  // zeros when there is no bias
                brow[4 * q] = bv.x, brow[4 * q + 1] = bv.y, brow[4 * q + 2] = bv.z, brow[4 * q + 3] = bv.w;
              }
              const bool relu_q = ea.relu != 0 && !(ea.out_inv_scale > 0.0f);
              if (ea.bias) {
                if (relu_q)
                  requant_block<true, true>(acc[0], mrow, brow, ea.out_inv_scale, packed);
                else
                  requant_block<true, false>(acc[0], mrow, brow, ea.out_inv_scale, packed);
              } else {
                if (relu_q)
                  requant_block<false, true>(acc[0], mrow, brow, ea.out_inv_scale, packed);
                else
                  requant_block<false, false>(acc[0], mrow, brow, ea.out_inv_scale, packed);
              }
            }
            if (MODE == 1 || whole) {
              // per-lane part of the address fixed for the whole pass, the rest scalar; pixels outside
              // the output get an offset beyond the buffer and are dropped
              const int s_off = s_tile + (8 * (wave >> 1) + 2 * bl) * s_row;
              __builtin_amdgcn_raw_buffer_store_b64((v2u){packed[0], packed[1]}, yr, (col_ok && oh < a.OH) ? lane_off : (int)0x80000000, s_off, 0);
            } else if (px_ok) {
              RMSMP_GLOBAL uint8_t* dst = as_global((uint8_t*)ea.Y) + n * row_bytes + (gpos0 >> 1);
              for (int b = 0; b < n_rows / 2; ++b) dst[b] = (uint8_t)(packed[b >> 2] >> (8 * (b & 3)));
            }
          }
        };
        // (mine_live is the same for the whole wave: every lane feeds the MFMAs)
        if constexpr (MODE == 1) {
          // All four blocks in one piece of straight-line code, software-pipelined: the MFMA chain of
          // block bl + 1 (seven dependent instructions, each waiting for the one before) is issued
          // between the vector instructions that requantize block bl, so the wave's matrix work runs
          // in the shadow of its own vector work (the waves of a SIMD pass the per-tile barrier
          // together and would otherwise all be in their MFMA chains, then all in their epilogues).
          if (mine_live) {
            auto frags = [&](const int bl, v4i (&bf)[KHW]) {
              const int oh_l = 8 * (wave >> 1) + 2 * bl + pr;
              const uint8_t* fp = buf + (oh_l * 2) * CF_ROWB + (pc + 2 * hh + pos.shift) * 8;
#pragma unroll
              for (int kh = 0; kh < KHW; ++kh) {
                const uint2 lo = *(const uint2*)(fp + kh * CF_ROWB);
                const uint2 hi = *(const uint2*)(fp + kh * CF_ROWB + 8);
                bf[kh] = (v4i){(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
              }
            };
            auto chain = [&](const v4i (&bf)[KHW]) -> v16i {
              v16i acc;
#pragma unroll
              for (int r = 0; r < 16; ++r) acc[r] = 0;
#pragma unroll
              for (int kh = 0; kh < KHW; ++kh) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(av[kh], bf[kh], acc, 0, 0, 0);
              return acc;
            };
            auto finish = [&](const int bl, const v16i& acc) {
              uint32_t packed[2];
              float brow[16];
              requant_block<false, false>(acc, mkeep, brow, ea.out_inv_scale, packed);
              const int oh = pos.oh0 + 8 * (wave >> 1) + 2 * bl + pr;
              const int s_off = s_tile + (8 * (wave >> 1) + 2 * bl) * s_row;
              __builtin_amdgcn_raw_buffer_store_b64((v2u){packed[0], packed[1]}, yr, (col_ok && oh < a.OH) ? lane_off : (int)0x80000000, s_off, 0);
            };
            v4i bf0[KHW], bf1[KHW];
            frags(0, bf0);
            v16i cur = chain(bf0);
            frags(1, bf1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int bl = 0; bl < 4; ++bl) {
              v16i nxt = cur;
              if (bl + 1 < 4) nxt = chain((bl & 1) ? bf0 : bf1);
              if (bl + 2 < 4) frags(bl + 2, (bl & 1) ? bf1 : bf0);
              finish(bl, cur);
              if (bl + 1 < 4) {
                // one MFMA of the next block's chain behind every dozen vector instructions of this block's epilogue
#pragma unroll
                for (int kh = 0; kh < KHW; ++kh) {
                  __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
                  __builtin_amdgcn_sched_group_barrier(0x002, 12, 0);  // VALU
                }
              }
              __builtin_amdgcn_sched_barrier(0);
              cur = nxt;
            }
          }
        } else {
#pragma unroll 1
          for (int bl = 0; bl < 4; ++bl) {
            if (!mine_live) break;
            do_block(bl);
          }
        }
        // ---- the next tile's pixels go to the other buffer (nobody reads it before the barrier)
        if (more) store_units(nxt, raw, buf0 + (cur ^ 1) * BUF);
        pos = nxt;
        __syncthreads();
      }
    };
    run_tiles(std::integral_constant<int, MODE_>{});
  }
}

static uint32_t cf_div_magic(int64_t d) {
  return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + (uint64_t)d - 1) / (uint64_t)d);
}

static bool conv_first_applies(const GemmArgs& a) {
  if (!(a.conv && a.w.k_layout == K_FILTER_ROWS && a.ep.act_bits == 8)) return false;
  if (a.ep.out_kind == 3) return false;  // the GELU epilogue lives in the general kernels
  if (a.d.C != 3 || a.d.stride != 2 || a.d.KH != a.d.KW) return false;
  if (!(a.d.KH == 3 || a.d.KH == 5 || a.d.KH == 7)) return false;
  if (!(a.d.pad == 1 || a.d.pad == 3)) return false;  // pixel pairs start on an odd pixel, at most 4 left of the image
  if (a.d.W % 4 != 0) return false;                          // input rows start on a dword
  if (a.w.nks < a.d.KH || a.w.n_tiles > CF_MAX_TILES) return false;
  const int64_t x_bytes = (int64_t)a.d.B * a.d.H * a.d.W * 3;
  if (x_bytes >= ((int64_t)1 << 31) || x_bytes < 16) return false;
  const int64_t tiles = (int64_t)a.d.B * ((a.OH + CF_T - 1) / CF_T) * ((a.OW + CF_T - 1) / CF_T);
  if (tiles >= ((int64_t)1 << 24)) return false;  // one-multiply division of tile numbers
  return true;
}

template <int KHW>
static int launch_conv_first_t(const GemmArgs& a, const FirstGeom& g, unsigned blocks, hipStream_t s) {
  constexpr int PH = 2 * (CF_T - 1) + KHW;
  const size_t lds = (size_t)2 * PH * CF_ROWB + (size_t)a.w.n_tiles * TILE_M * (16 + 8);  // at most 12 + 48 KiB
  // which of the three pixel-tile loops the launch needs (see the kernel)
  const int64_t row_bytes = a.M / 2;
  const bool relu_step = a.ep.relu != 0 && !(a.ep.out_inv_scale > 0.0f);
  const bool u4_plain = a.ep.out_kind == 2 && a.ep.act_zero_point == 0 && a.N * row_bytes < ((int64_t)1 << 31);
  // every lane of the lean loop stores 16 whole codes: full weight tiles, 8-byte aligned places
  const bool all_whole = a.M % TILE_M == 0 && (((uintptr_t)a.Y) & 7) == 0;
  if (u4_plain && a.ep.bias == nullptr && !relu_step && all_whole)
    hipLaunchKernelGGL((conv_first_kernel<KHW, 1>), dim3(blocks), dim3(256), lds, s, a, g);
  else if (u4_plain)
    hipLaunchKernelGGL((conv_first_kernel<KHW, 2>), dim3(blocks), dim3(256), lds, s, a, g);
  else
    hipLaunchKernelGGL((conv_first_kernel<KHW, 0>), dim3(blocks), dim3(256), lds, s, a, g);
  return (int)hipGetLastError();
}

// Launches the first-layer kernel when the layer fits it; *applied says whether it did.
int try_launch_conv_first(const GemmArgs& a, void* stream, bool* applied) {
  *applied = conv_first_applies(a);
  if (!*applied) return 0;
  last_dispatch() = DispatchRecord{4, 0, 0, 0, 0};
  FirstGeom g;
  g.tiles_w = (a.OW + CF_T - 1) / CF_T;
  g.tiles_h = (a.OH + CF_T - 1) / CF_T;
  g.total_tiles = a.d.B * g.tiles_w * g.tiles_h;
  // Three work-groups share a compute unit (register budget): exactly that many work-groups when
  // there are enough tiles, the tiles spread evenly over them, so that every compute unit carries
  // the same load in one round and a work-group spreads its weight fetch over several tiles.
  int n_wg = g.total_tiles < 768 ? g.total_tiles : 768;
  g.tiles_base = g.total_tiles / n_wg;
  g.tiles_rem = g.total_tiles % n_wg;
  g.magic_tw = cf_div_magic(g.tiles_w);
  g.magic_thw = cf_div_magic((int64_t)g.tiles_w * g.tiles_h);
  const unsigned blocks = (unsigned)n_wg;
  hipStream_t s = (hipStream_t)stream;
  switch (a.d.KH) {
    case 3: return launch_conv_first_t<3>(a, g, blocks, s);
    case 5: return launch_conv_first_t<5>(a, g, blocks, s);
    default: return launch_conv_first_t<7>(a, g, blocks, s);
  }
}

}  // namespace rmsmp
