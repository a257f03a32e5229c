// Internal declarations shared by the host packer, the kernels and the C-ABI glue.
// Not installed; the public interface is include/rmsmp.h.
#pragma once
#include <atomic>
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "rmsmp.h"

namespace rmsmp {

// A weight tile is TILE_M rows of one storage class; the K axis is cut in steps of KSTEP
// elements, the depth of one v_mfma_i32_32x32x32_i8 (the int8 MFMA shape that runs at the full
// rate on gfx950; 16x16x64 runs at half of it).  K is padded to a multiple of KPAD_UNIT.
constexpr int TILE_M = 32;
constexpr int KSTEP = 32;
constexpr int KPAD_UNIT = 64;
constexpr int LANES = 64;

// MFMA row i of a tile holds the row at grouped offset tile_row_goff(i): with this order the
// 16 accumulator registers of a lane are 16 consecutive grouped rows (lanes 0..31 rows 0..15,
// lanes 32..63 rows 16..31), so a lane can emit its 4-bit output codes as one 8-byte store.
constexpr int tile_row_goff(int i) { return 16 * ((i / 4) % 2) + 4 * (i / 8) + i % 4; }

// Order of the internal (stored) K axis.
enum KLayout : int32_t {
  // (tap, input-channel position): K = taps * C, padded at the end.  Plain GEMMs have one tap.
  K_TAP_CHANNEL = 0,
  // Layers with at most four input channels and a square KW x KW filter, KW <= 8 (a network's
  // first layer): one K step per filter row, element (kh, kw, c) at kh*32 + kw*4 + c, zero
  // weights where kw >= KW or c >= C.  A filter row of an NHWC image whose pixels are padded to
  // four bytes is then one aligned 32-byte run, and no im2col matrix has to be built.
  K_FILTER_ROWS = 1
};

// How a tile's codes are stored and decoded in registers.
enum TileKind : int32_t {
  TILE_NIB_SHIFT = 0,  // 4-bit two's-complement codes; decode = mask/shift, yields 16*q
  TILE_NIB_LUT = 1,    // 4-bit codes through a per-row 16-entry byte table (PoT-4 exponent codes)
  TILE_I8 = 2          // 8-bit codes, no decode (Fixed-8)
};

struct TileDesc {
  int32_t kind;      // TileKind
  int32_t nvalid;    // rows of the tile that are real (the rest is zero padding)
  int32_t g0;        // grouped position of the tile's first row
  int32_t reserved;
  int64_t blob_off;  // byte offset of the tile in the blob
};

// Within a run of 16 consecutive K elements the MFMA operand slot s holds element kSlot[s]:
// the order that mask/shift nibble extraction produces (even elements of each 8, then odd).
constexpr int kSlot[16] = {0, 2, 4, 6, 1, 3, 5, 7, 8, 10, 12, 14, 9, 11, 13, 15};

struct HostPacked {
  int64_t M = 0, K = 0, C = 0;
  int32_t taps = 1;
  int32_t k_layout = 0;            // KLayout of the internal K axis
  int64_t Kpad = 0, nks = 0;
  int64_t counts[3] = {0, 0, 0};
  std::vector<int32_t> perm;       // [M] grouped position -> original row
  std::vector<float> rowscale;     // [M] original order
  std::vector<int32_t> rowsum;     // [M] original order
  std::vector<uint8_t> scheme;     // [M] original order
  std::vector<int32_t> kmap;       // [Kpad] internal k -> original k, -1 = zero padding
  std::vector<TileDesc> tiles;
  // tables indexed by padded grouped row p = tile*TILE_M + grouped offset
  std::vector<float> p_rowscale;
  std::vector<int32_t> p_rowsum, p_orig, p_gpos;
  std::vector<uint32_t> p_lut;     // 4 words per padded row
  std::vector<int32_t> p_meta;     // 4 words per padded row: rowscale bits, rowsum, original row (-1 = padding), grouped position
  std::vector<uint8_t> blob;
};

// Host side of rmsmp_pack_weights: quantize, encode, group, lay out.  Returns RMSMP_OK or an
// error with `err` filled.
rmsmp_status pack_host(const float* W, int64_t M, int64_t K, const uint8_t* scheme, const float* alpha,
                       int32_t taps, const int32_t* in_perm, HostPacked* out, std::string* err, uint32_t flags = 0);

// Decode a blob (as laid out by pack_host) back to integer weights in original order.
void unpack_host(const HostPacked& hp, const uint8_t* blob, int8_t* wint);

rmsmp_status ratio_counts(int64_t M, int32_t a, int32_t b, int32_t c, int64_t counts[3]);
rmsmp_status assign_by_variance(const float* W, int64_t M, int64_t K, int64_t n_pot4, uint8_t* scheme);

// Device-side view handed to the kernels.
struct DevicePacked {
  const uint8_t* blob = nullptr;
  const TileDesc* tiles = nullptr;
  const int32_t* p_meta = nullptr;  // per padded row: {rowscale bits, rowsum, original row or -1, grouped position}
  const uint32_t* p_lut = nullptr;
  int32_t n_tiles = 0;
  int32_t nks = 0;
  int32_t k_layout = 0;  // KLayout
  // Tiles are ordered by class (TileKind 0, 1, 2) and all tiles of a class have the same size,
  // so a kernel finds a tile's class, blob offset and live row count from these six numbers
  // without touching memory.
  int32_t class_tiles[3] = {0, 0, 0};
  int32_t class_rows[3] = {0, 0, 0};
};

// Where weight tile mt lives, computed from DevicePacked alone.
struct TileRef {
  int kind;
  int nvalid;
  int64_t blob_off;
};

// Break points of the GELU + affine 4-bit code as a function of the fp32 pre-activation y
// (gelu_host.cpp).  Rising branch (y >= y_split): code = max{ c : rise[c] <= y }; the kernels start
// from the code y itself would get, which is never below and at most fix_steps above.  Falling
// branch (y < y_split): code = fall_base + #{ j < n_fall : y <= fall[j] }.
struct GeluTable {
  float rise[16];
  float fall[16];
  float y_split;
  int32_t fix_steps, fall_base, n_fall;
};
void gelu_table(float inv_s, int32_t zero_point, GeluTable* t);

struct GemmArgs {
  DevicePacked w;
  int64_t M = 0, K = 0, N = 0;
  const void* X = nullptr;
  void* Y = nullptr;
  rmsmp_epilogue ep{};
  // convolution (implicit im2col); conv == 0 for a plain GEMM
  int32_t conv = 0;
  rmsmp_conv_desc d{};
  int32_t OH = 0, OW = 0;
  // out_kind 3 only; kept last so that the other epilogues never fetch it
  GeluTable gelu{};
};

struct Im2colArgs {
  const void* X = nullptr;
  void* cols = nullptr;  // [N][Kpad/2] (4-bit) or [N][Kpad] (8-bit), internal K order
  rmsmp_conv_desc d{};
  int32_t OH = 0, OW = 0;
  int64_t N = 0, K = 0, Kpad = 0;
  int32_t act_bits = 4;
  int32_t zero_point = 0;
  int32_t k_layout = 0;  // KLayout of the columns to produce
};

// Quantization-aware-training helpers (fakequant.hip); every pointer is a device pointer.
struct FakeQuantArgs {
  const float* W = nullptr;       // [M][K]
  const uint8_t* scheme = nullptr;  // [M]
  const float* alpha = nullptr;   // [M] or null: per-row maximum
  float* What = nullptr;          // [M][K]
  float* alpha_out = nullptr;     // [M] or null
  int64_t M = 0, K = 0;
};
struct SteArgs {
  const float* W = nullptr;      // [M][K], read only when alpha is given
  const float* alpha = nullptr;  // [M] or null
  const float* dWhat = nullptr;  // [M][K]
  float* dW = nullptr;           // [M][K]
  int64_t M = 0, K = 0;
};
int launch_fake_quant_rows(const FakeQuantArgs& a, void* stream);
int launch_ste_backward(const SteArgs& a, void* stream);

// Test hooks.  forced_split(): a wave split {pixel blocks per wave, K split, pixel blocks side by
// side, tile pairs} the LDS-resident kernel should use where it fits the layer (all zero:
// automatic); like last_dispatch() it belongs to the calling thread.
// last_dispatch(): which kernel the calling thread's last launch_gemm went to.
struct DispatchRecord {
  int kernel = 0;  // 0 none, 1 general, 2 skinny, 3 small-channel rows, 4 first layer, 5 LDS-resident, 6 LDS-resident, two layers in one launch
  int xb = 0, ks = 0, nwt = 0, ms = 0;
};
int* forced_split();
DispatchRecord& last_dispatch();

// Kernel launchers (kernels.hip).  Return hipError_t as int.
int launch_gemm(const GemmArgs& a, void* stream);
// LDS-resident implicit-im2col kernel (patch_wide.hip): launches when the layer fits it and says
// so in *applied.
int try_launch_wide(const GemmArgs& a, void* stream, bool* applied);
// The same kernel for two layers that read one input (a 3x3 and a 1x1 layer), as one launch.
int try_launch_wide_pair(const GemmArgs& a, const GemmArgs& b, void* stream, bool* applied);
// First-layer kernel (conv_first.hip): 3 input channels, 8-bit activations, stride 2; same convention.
int try_launch_conv_first(const GemmArgs& a, void* stream, bool* applied);
int launch_im2col(const Im2colArgs& a, void* stream);
// Machine rates (peaks.hip): MFMA-only int8 TOP/s and copy GB/s (read + written) of the current device.
int measure_peaks(double* mfma_tops, double* copy_gbs);

// Dynamic LDS above 64 KiB must be allowed per kernel once on every device.  `done` is the
// kernel's own bit mask of devices that have it (one per launcher, a function-local static):
// two threads that race on the first launch both set the attribute, which is harmless.
int allow_large_lds(const void* kernel, std::atomic<uint64_t>& done);

}  // namespace rmsmp

struct rmsmp_packed {
  rmsmp::HostPacked host;
  rmsmp::DevicePacked dev;
  void* dev_alloc = nullptr;  // one allocation holding every device table
  size_t dev_bytes = 0;
  int device = 0;
};
