// C-ABI glue of librmsmp: argument checking, device memory of packed layers, kernel dispatch.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstring>
#include <new>
#include <string>

#include "rmsmp_internal.h"

namespace {

thread_local std::string g_err;

rmsmp_status fail(rmsmp_status s, const std::string& msg) {
  g_err = msg;
  return s;
}

rmsmp_status hip_fail(hipError_t e, const char* what) {
  g_err = std::string(what) + ": " + hipGetErrorString(e);
  return RMSMP_EHIP;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Workspace of rmsmp_conv2d_static_workspace.  In host code the array's name is only a handle
// for hipGetSymbolAddress, never an address: kernels get the pointer that call returns for the
// device they run on (each GPU has its own copy of the array at its own address).
static __device__ __align__(256) uint8_t scratch[RMSMP_STATIC_WORKSPACE_BYTES];
std::atomic<void*> g_scratch_ptr[64];

rmsmp_status static_workspace(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= 64) return fail(RMSMP_EUNSUPPORTED, "static workspace: device ordinal above 63");
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(static workspace)");
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return RMSMP_OK;
}

rmsmp_status check_epilogue(const rmsmp_epilogue* ep, int64_t M) {
  if (!ep) return fail(RMSMP_EINVAL, "epilogue is NULL");
  if (ep->act_bits != 4 && ep->act_bits != 8) return fail(RMSMP_EINVAL, "act_bits must be 4 or 8");
  if (ep->out_kind < 0 || ep->out_kind > 3) return fail(RMSMP_EINVAL, "out_kind must be 0, 1, 2 or 3");
  if (ep->out_kind == 3) {
    if (ep->relu != 0) return fail(RMSMP_EINVAL, "out_kind 3 applies GELU: relu must be 0");
    if (!(ep->out_inv_scale > 0.0f) || !std::isfinite(ep->out_inv_scale))
      return fail(RMSMP_EINVAL, "out_kind 3 needs a positive, finite out_inv_scale");
    if (ep->out_zero_point < 0 || ep->out_zero_point > 15) return fail(RMSMP_EINVAL, "out_zero_point must be in 0..15");
  }
  if (ep->relu != 0 && ep->relu != 1) return fail(RMSMP_EINVAL, "relu must be 0 or 1");
  if (ep->act_bits == 4 && (ep->act_zero_point < 0 || ep->act_zero_point > 15))
    return fail(RMSMP_EINVAL, "act_zero_point must be in 0..15 for 4-bit codes");
  if (ep->act_bits == 8 && (ep->act_zero_point < -128 || ep->act_zero_point > 127))
    return fail(RMSMP_EINVAL, "act_zero_point must be in -128..127 for 8-bit codes");
  if (ep->out_kind >= 2 && (M & 1)) return fail(RMSMP_ESHAPE, "4-bit output needs an even number of rows");
  return RMSMP_OK;
}

// Break points of the GELU epilogue for the scale and zero point of this call; the last pair a
// thread asked for is kept, so a serving loop with fixed scales pays for the bisection once.
void fill_gelu_table(const rmsmp_epilogue& ep, rmsmp::GemmArgs* a) {
  if (ep.out_kind != 3) return;
  thread_local float cached_inv = 0.0f;
  thread_local int32_t cached_z = -1;
  thread_local rmsmp::GeluTable cached;
  if (cached_inv != ep.out_inv_scale || cached_z != ep.out_zero_point) {
    rmsmp::gelu_table(ep.out_inv_scale, ep.out_zero_point, &cached);
    cached_inv = ep.out_inv_scale;
    cached_z = ep.out_zero_point;
  }
  a->gelu = cached;
}

}  // namespace

extern "C" {

const char* rmsmp_last_error(void) { return g_err.c_str(); }

const char* rmsmp_version(void) { return "librmsmp 0.1 (gfx950)"; }

rmsmp_status rmsmp_ratio_counts(int64_t M, int32_t pct_pot4, int32_t pct_fixed4, int32_t pct_fixed8,
                                int64_t counts[3]) {
  rmsmp_status s = rmsmp::ratio_counts(M, pct_pot4, pct_fixed4, pct_fixed8, counts);
  if (s != RMSMP_OK) return fail(s, "ratio_counts: percentages must be non-negative and sum to 100");
  return s;
}

rmsmp_status rmsmp_assign_by_variance(const float* W, int64_t M, int64_t K, int64_t n_pot4, uint8_t* scheme) {
  rmsmp_status s = rmsmp::assign_by_variance(W, M, K, n_pot4, scheme);
  if (s != RMSMP_OK) return fail(s, "assign_by_variance: bad argument");
  return s;
}

rmsmp_status rmsmp_pack_weights(const float* W, int64_t M, int64_t K, const uint8_t* scheme, const float* alpha,
                                int32_t taps, const int32_t* in_perm, rmsmp_packed** out) {
  return rmsmp_pack_weights_opt(W, M, K, scheme, alpha, taps, in_perm, 0u, out);
}

rmsmp_status rmsmp_pack_weights_opt(const float* W, int64_t M, int64_t K, const uint8_t* scheme, const float* alpha,
                                    int32_t taps, const int32_t* in_perm, uint32_t flags, rmsmp_packed** out) {
  if (!out) return fail(RMSMP_EINVAL, "pack_weights: out is NULL");
  if (flags & ~RMSMP_PACK_POT_AS_INT8) return fail(RMSMP_EINVAL, "pack_weights: unknown flag");
  *out = nullptr;
  rmsmp_packed* p = new (std::nothrow) rmsmp_packed();
  if (!p) return fail(RMSMP_ENOMEM, "pack_weights: host allocation failed");
  std::string err;
  rmsmp_status st;
  try {
    st = rmsmp::pack_host(W, M, K, scheme, alpha, taps, in_perm, &p->host, &err, flags);
  } catch (const std::bad_alloc&) {
    delete p;
    return fail(RMSMP_ENOMEM, "pack_weights: host allocation failed");
  }
  if (st != RMSMP_OK) {
    delete p;
    return fail(st, err);
  }
  const rmsmp::HostPacked& h = p->host;
  // one device allocation: blob | tiles | row metadata | lut
  const size_t n_blob = align_up(h.blob.size(), 256);
  const size_t n_tiles = align_up(h.tiles.size() * sizeof(rmsmp::TileDesc), 256);
  const size_t n_meta = align_up(h.p_meta.size() * 4, 256);
  const size_t n_lut = align_up(h.p_lut.size() * 4, 256);
  const size_t total = n_blob + n_tiles + n_meta + n_lut;
  hipError_t e = hipGetDevice(&p->device);
  if (e != hipSuccess) {
    delete p;
    return hip_fail(e, "hipGetDevice");
  }
  e = hipMalloc(&p->dev_alloc, total);
  if (e != hipSuccess) {
    delete p;
    g_err = std::string("pack_weights: hipMalloc: ") + hipGetErrorString(e);
    return RMSMP_ENOMEM;
  }
  p->dev_bytes = total;
  uint8_t* base = (uint8_t*)p->dev_alloc;
  size_t off = 0;
  auto put = [&](const void* src, size_t bytes, size_t reserved) -> const uint8_t* {
    uint8_t* dst = base + off;
    if (bytes && e == hipSuccess) e = hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice);
    off += reserved;
    return dst;
  };
  p->dev.blob = put(h.blob.data(), h.blob.size(), n_blob);
  p->dev.tiles = (const rmsmp::TileDesc*)put(h.tiles.data(), h.tiles.size() * sizeof(rmsmp::TileDesc), n_tiles);
  p->dev.p_meta = (const int32_t*)put(h.p_meta.data(), h.p_meta.size() * 4, n_meta);
  p->dev.p_lut = (const uint32_t*)put(h.p_lut.data(), h.p_lut.size() * 4, n_lut);
  p->dev.n_tiles = (int32_t)h.tiles.size();
  p->dev.nks = (int32_t)h.nks;
  p->dev.k_layout = h.k_layout;
  for (const auto& t : h.tiles) {
    p->dev.class_tiles[t.kind] += 1;
    p->dev.class_rows[t.kind] += t.nvalid;
  }
  if (e != hipSuccess) {
    (void)hipFree(p->dev_alloc);
    delete p;
    return hip_fail(e, "pack_weights: hipMemcpy");
  }
  // the host copy of the blob is not needed any more
  std::vector<uint8_t>().swap(p->host.blob);
  *out = p;
  return RMSMP_OK;
}

rmsmp_status rmsmp_pack_roundtrip_host(const float* W, int64_t M, int64_t K, const uint8_t* scheme,
                                       const float* alpha, int32_t taps, const int32_t* in_perm, int8_t* wint,
                                       float* rowscale, int32_t* rowsum, int32_t* perm) {
  rmsmp::HostPacked h;
  std::string err;
  rmsmp_status st;
  try {
    st = rmsmp::pack_host(W, M, K, scheme, alpha, taps, in_perm, &h, &err);
  } catch (const std::bad_alloc&) {
    return fail(RMSMP_ENOMEM, "pack_roundtrip_host: host allocation failed");
  }
  if (st != RMSMP_OK) return fail(st, err);
  if (wint) {
    std::memset(wint, 0, (size_t)M * (size_t)K);
    rmsmp::unpack_host(h, h.blob.data(), wint);
  }
  if (rowscale) std::memcpy(rowscale, h.rowscale.data(), (size_t)M * 4);
  if (rowsum) std::memcpy(rowsum, h.rowsum.data(), (size_t)M * 4);
  if (perm) std::memcpy(perm, h.perm.data(), (size_t)M * 4);
  return RMSMP_OK;
}

void rmsmp_free_packed(rmsmp_packed* p) {
  if (!p) return;
  if (p->dev_alloc) (void)hipFree(p->dev_alloc);
  delete p;
}

rmsmp_status rmsmp_packed_info(const rmsmp_packed* p, int64_t* M, int64_t* K, int64_t counts[3],
                               const int32_t** perm, const float** rowscale, const int32_t** rowsum) {
  if (!p) return fail(RMSMP_EINVAL, "packed_info: NULL handle");
  if (M) *M = p->host.M;
  if (K) *K = p->host.K;
  if (counts)
    for (int i = 0; i < 3; ++i) counts[i] = p->host.counts[i];
  if (perm) *perm = p->host.perm.data();
  if (rowscale) *rowscale = p->host.rowscale.data();
  if (rowsum) *rowsum = p->host.rowsum.data();
  return RMSMP_OK;
}

rmsmp_status rmsmp_unpack_codes(const rmsmp_packed* p, int8_t* wint) {
  if (!p || !wint) return fail(RMSMP_EINVAL, "unpack_codes: NULL argument");
  size_t blob_bytes = 0;
  for (const auto& t : p->host.tiles)
    blob_bytes += (size_t)p->host.nks * rmsmp::LANES * (t.kind == rmsmp::TILE_I8 ? 16 : 8);
  std::vector<uint8_t> blob;
  try {
    blob.resize(blob_bytes);
  } catch (const std::bad_alloc&) {
    return fail(RMSMP_ENOMEM, "unpack_codes: host allocation failed");
  }
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess && blob_bytes) e = hipMemcpy(blob.data(), p->dev.blob, blob_bytes, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_fail(e, "unpack_codes: hipMemcpy");
  std::memset(wint, 0, (size_t)p->host.M * (size_t)p->host.K);
  rmsmp::unpack_host(p->host, blob.data(), wint);
  return RMSMP_OK;
}

rmsmp_status rmsmp_gemm(const rmsmp_packed* Wp, const void* X, int64_t N, const rmsmp_epilogue* ep, void* Y,
                        void* stream) {
  if (!Wp) return fail(RMSMP_EINVAL, "gemm: NULL packed weights");
  rmsmp_status st = check_epilogue(ep, Wp->host.M);
  if (st != RMSMP_OK) return st;
  if (N < 0) return fail(RMSMP_ESHAPE, "gemm: N < 0");
  if (N == 0) return RMSMP_OK;
  if (!X || !Y) return fail(RMSMP_EINVAL, "gemm: NULL X or Y");
  if (Wp->host.k_layout != rmsmp::K_TAP_CHANNEL)
    return fail(RMSMP_EUNSUPPORTED, "gemm: these weights are stored for a small-channel convolution; use rmsmp_conv2d");
  if (ep->act_bits == 4 && (Wp->host.K & 1)) return fail(RMSMP_ESHAPE, "gemm: 4-bit activations need an even K");
  if (((uintptr_t)X & 15) != 0) return fail(RMSMP_EINVAL, "gemm: X must be 16-byte aligned");
  if (N > (int64_t)0x7fffffff * 64) return fail(RMSMP_ESHAPE, "gemm: N too large");
  rmsmp::GemmArgs a;
  a.w = Wp->dev;
  a.M = Wp->host.M;
  a.K = Wp->host.K;
  a.N = N;
  a.X = X;
  a.Y = Y;
  a.ep = *ep;
  a.conv = 0;
  fill_gelu_table(*ep, &a);
  hipError_t e = (hipError_t)rmsmp::launch_gemm(a, stream);
  if (e != hipSuccess) return hip_fail(e, "gemm: kernel launch");
  return RMSMP_OK;
}

static rmsmp_status conv_geometry(const rmsmp_packed* Wp, const rmsmp_conv_desc* d, int32_t act_bits, int* OH,
                                  int* OW) {
  if (!Wp || !d) return fail(RMSMP_EINVAL, "conv2d: NULL argument");
  if (d->B < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->KH < 1 || d->KW < 1 || d->stride < 1 || d->pad < 0)
    return fail(RMSMP_ESHAPE, "conv2d: bad geometry");
  if ((int64_t)d->C * d->KH * d->KW != Wp->host.K || d->KH * d->KW != Wp->host.taps)
    return fail(RMSMP_ESHAPE, "conv2d: C*KH*KW and KH*KW must match the packed layer's K and taps");
  if (act_bits == 4 && (d->C & 1)) return fail(RMSMP_ESHAPE, "conv2d: 4-bit activations need an even C");
  if (Wp->host.k_layout == rmsmp::K_FILTER_ROWS && d->KH != d->KW)
    return fail(RMSMP_EUNSUPPORTED, "conv2d: layers with at most 4 input channels are stored for square filters");
  const int oh = (d->H + 2 * d->pad - d->KH) / d->stride + 1;
  const int ow = (d->W + 2 * d->pad - d->KW) / d->stride + 1;
  if (d->H + 2 * d->pad < d->KH || d->W + 2 * d->pad < d->KW || oh < 1 || ow < 1)
    return fail(RMSMP_ESHAPE, "conv2d: empty output");
  *OH = oh;
  *OW = ow;
  return RMSMP_OK;
}

// im2col is done on the fly whenever a 16-channel chunk is one aligned load
// Which path a convolution takes.  Implicit: the kernels address the NHWC input themselves (any
// layer whose channel count is a multiple of 16, and 8-bit small-channel layers stored with one
// K step per filter row).  Otherwise the lowered matrix is written to the caller's workspace.
static bool conv_is_implicit(const rmsmp_packed* Wp, const rmsmp_conv_desc* d, int32_t act_bits) {
  if (Wp->host.k_layout == rmsmp::K_FILTER_ROWS) return act_bits == 8 && d->stride <= 8;
  return d->C % 16 == 0;
}

rmsmp_status rmsmp_debug_set_wave_split(int32_t pixel_blocks, int32_t k_split, int32_t side_by_side, int32_t tile_pairs) {
  if (pixel_blocks < 0 || k_split < 0 || side_by_side < 0 || tile_pairs < 0)
    return fail(RMSMP_EINVAL, "debug_set_wave_split: negative value");
  int* split = rmsmp::forced_split();
  split[0] = pixel_blocks;
  split[1] = k_split;
  split[2] = side_by_side;
  split[3] = tile_pairs;
  return RMSMP_OK;
}

rmsmp_status rmsmp_debug_last_dispatch(int32_t out[5]) {
  if (!out) return fail(RMSMP_EINVAL, "debug_last_dispatch: NULL out");
  const rmsmp::DispatchRecord& r = rmsmp::last_dispatch();
  out[0] = r.kernel, out[1] = r.xb, out[2] = r.ks, out[3] = r.nwt, out[4] = r.ms;
  return RMSMP_OK;
}

rmsmp_status rmsmp_debug_gelu_breakpoints(float out_inv_scale, int32_t out_zero_point, float rise[16], float fall[16],
                                          float* y_split, int32_t* fall_base, int32_t* n_fall) {
  if (!rise || !fall || !y_split || !fall_base || !n_fall) return fail(RMSMP_EINVAL, "debug_gelu_breakpoints: NULL output");
  if (!(out_inv_scale > 0.0f) || !std::isfinite(out_inv_scale) || out_zero_point < 0 || out_zero_point > 15)
    return fail(RMSMP_EINVAL, "debug_gelu_breakpoints: scale must be positive and finite, zero point in 0..15");
  rmsmp::GeluTable t;
  rmsmp::gelu_table(out_inv_scale, out_zero_point, &t);
  std::memcpy(rise, t.rise, sizeof(t.rise));
  std::memcpy(fall, t.fall, sizeof(t.fall));
  *y_split = t.y_split;
  *fall_base = t.fall_base;
  *n_fall = t.n_fall;
  return RMSMP_OK;
}

rmsmp_status rmsmp_debug_measure_peaks(double* mfma_int8_tops, double* copy_gbs) {
  hipError_t e = (hipError_t)rmsmp::measure_peaks(mfma_int8_tops, copy_gbs);
  if (e != hipSuccess) return hip_fail(e, "debug_measure_peaks");
  return RMSMP_OK;
}

rmsmp_status rmsmp_conv2d_workspace_size(const rmsmp_packed* Wp, const rmsmp_conv_desc* d, int32_t act_bits,
                                         size_t* bytes) {
  if (!bytes) return fail(RMSMP_EINVAL, "conv2d_workspace_size: NULL bytes");
  if (act_bits != 4 && act_bits != 8) return fail(RMSMP_EINVAL, "act_bits must be 4 or 8");
  int OH, OW;
  rmsmp_status st = conv_geometry(Wp, d, act_bits, &OH, &OW);
  if (st != RMSMP_OK) return st;
  if (conv_is_implicit(Wp, d, act_bits)) {
    *bytes = 0;
    return RMSMP_OK;
  }
  const size_t N = (size_t)d->B * OH * OW;
  const size_t row = act_bits == 4 ? (size_t)Wp->host.Kpad / 2 : (size_t)Wp->host.Kpad;
  *bytes = align_up(N * row, 256);
  return RMSMP_OK;
}

rmsmp_status rmsmp_conv2d(const rmsmp_packed* Wp, const void* X, const rmsmp_conv_desc* d,
                          const rmsmp_epilogue* ep, void* Y, void* workspace, size_t workspace_bytes,
                          void* stream) {
  if (!Wp) return fail(RMSMP_EINVAL, "conv2d: NULL packed weights");
  rmsmp_status st = check_epilogue(ep, Wp->host.M);
  if (st != RMSMP_OK) return st;
  int OH, OW;
  st = conv_geometry(Wp, d, ep->act_bits, &OH, &OW);
  if (st != RMSMP_OK) return st;
  if (!X || !Y) return fail(RMSMP_EINVAL, "conv2d: NULL X or Y");
  if (((uintptr_t)X & 15) != 0) return fail(RMSMP_EINVAL, "conv2d: X must be 16-byte aligned");
  const int64_t N = (int64_t)d->B * OH * OW;
  rmsmp::GemmArgs a;
  a.w = Wp->dev;
  a.M = Wp->host.M;
  a.N = N;
  a.Y = Y;
  a.ep = *ep;
  a.d = *d;
  a.OH = OH;
  a.OW = OW;
  fill_gelu_table(*ep, &a);
  if (conv_is_implicit(Wp, d, ep->act_bits)) {
    a.K = Wp->host.K;
    a.X = X;
    a.conv = 1;
  } else {
    size_t need = 0;
    st = rmsmp_conv2d_workspace_size(Wp, d, ep->act_bits, &need);
    if (st != RMSMP_OK) return st;
    if (!workspace || workspace_bytes < need)
      return fail(RMSMP_EWORKSPACE, "conv2d: workspace of " + std::to_string(need) + " bytes required");
    if (((uintptr_t)workspace & 15) != 0) return fail(RMSMP_EINVAL, "conv2d: workspace must be 16-byte aligned");
    rmsmp::Im2colArgs ia;
    ia.X = X;
    ia.cols = workspace;
    ia.d = *d;
    ia.OH = OH;
    ia.OW = OW;
    ia.N = N;
    ia.K = Wp->host.K;
    ia.Kpad = Wp->host.Kpad;
    ia.act_bits = ep->act_bits;
    ia.zero_point = ep->act_zero_point;
    ia.k_layout = Wp->host.k_layout;
    hipError_t e = (hipError_t)rmsmp::launch_im2col(ia, stream);
    if (e != hipSuccess) return hip_fail(e, "conv2d: im2col launch");
    a.K = Wp->host.Kpad;
    a.X = workspace;
    a.conv = 0;
  }
  hipError_t e = (hipError_t)rmsmp::launch_gemm(a, stream);
  if (e != hipSuccess) return hip_fail(e, "conv2d: kernel launch");
  return RMSMP_OK;
}

// Both layers are checked as rmsmp_conv2d checks them; then one launch if the pair kernel takes
// them, else the two layers one after the other.
rmsmp_status rmsmp_conv2d_pair(const rmsmp_packed* WpA, const rmsmp_conv_desc* dA, const rmsmp_epilogue* epA, void* YA,
                               const rmsmp_packed* WpB, const rmsmp_conv_desc* dB, const rmsmp_epilogue* epB, void* YB,
                               const void* X, void* stream) {
  if (!WpA || !WpB) return fail(RMSMP_EINVAL, "conv2d_pair: NULL packed weights");
  if (!dA || !dB) return fail(RMSMP_EINVAL, "conv2d_pair: NULL convolution descriptor");
  if (dA->B != dB->B || dA->C != dB->C || dA->H != dB->H || dA->W != dB->W)
    return fail(RMSMP_ESHAPE, "conv2d_pair: the two layers must read the same input tensor (B, C, H, W)");
  if (!epA || !epB) return fail(RMSMP_EINVAL, "epilogue is NULL");
  if (epA->act_bits != epB->act_bits || epA->act_zero_point != epB->act_zero_point || epA->act_scale != epB->act_scale)
    return fail(RMSMP_EINVAL, "conv2d_pair: the two layers must agree on the input's scale, zero point and width");
  if (YA == YB && YA) return fail(RMSMP_EINVAL, "conv2d_pair: the two outputs must be different buffers");
  const rmsmp_packed* Wp[2] = {WpA, WpB};
  const rmsmp_conv_desc* d[2] = {dA, dB};
  const rmsmp_epilogue* ep[2] = {epA, epB};
  void* Y[2] = {YA, YB};
  rmsmp::GemmArgs a[2];
  for (int i = 0; i < 2; ++i) {
    rmsmp_status st = check_epilogue(ep[i], Wp[i]->host.M);
    if (st != RMSMP_OK) return st;
    int OH, OW;
    st = conv_geometry(Wp[i], d[i], ep[i]->act_bits, &OH, &OW);
    if (st != RMSMP_OK) return st;
    if (!X || !Y[i]) return fail(RMSMP_EINVAL, "conv2d_pair: NULL X or Y");
    if (((uintptr_t)X & 15) != 0) return fail(RMSMP_EINVAL, "conv2d_pair: X must be 16-byte aligned");
    if (!conv_is_implicit(Wp[i], d[i], ep[i]->act_bits))
      return fail(RMSMP_EWORKSPACE, "conv2d_pair: a layer that needs an im2col workspace cannot be part of a pair; use rmsmp_conv2d");
    a[i].w = Wp[i]->dev;
    a[i].M = Wp[i]->host.M;
    a[i].K = Wp[i]->host.K;
    a[i].N = (int64_t)d[i]->B * OH * OW;
    a[i].X = X;
    a[i].Y = Y[i];
    a[i].ep = *ep[i];
    a[i].d = *d[i];
    a[i].OH = OH;
    a[i].OW = OW;
    a[i].conv = 1;
    fill_gelu_table(*ep[i], &a[i]);
  }
  bool fused = false;
  hipError_t e = (hipError_t)rmsmp::try_launch_wide_pair(a[0], a[1], stream, &fused);
  if (e != hipSuccess) return hip_fail(e, "conv2d_pair: kernel launch");
  if (fused) return RMSMP_OK;
  for (int i = 0; i < 2; ++i) {
    e = (hipError_t)rmsmp::launch_gemm(a[i], stream);
    if (e != hipSuccess) return hip_fail(e, "conv2d_pair: kernel launch");
  }
  return RMSMP_OK;
}

rmsmp_status rmsmp_init(void) {
  void* ws = nullptr;
  return static_workspace(&ws);
}

rmsmp_status rmsmp_conv2d_static_workspace(const rmsmp_packed* Wp, const void* X, const rmsmp_conv_desc* d,
                                           const rmsmp_epilogue* ep, void* Y, void* stream) {
  if (!Wp) return fail(RMSMP_EINVAL, "conv2d: NULL packed weights");
  if (!ep) return fail(RMSMP_EINVAL, "epilogue is NULL");
  size_t need = 0;
  rmsmp_status st = rmsmp_conv2d_workspace_size(Wp, d, ep->act_bits, &need);
  if (st != RMSMP_OK) return st;
  if (need == 0) return rmsmp_conv2d(Wp, X, d, ep, Y, nullptr, 0, stream);
  if (need > (size_t)RMSMP_STATIC_WORKSPACE_BYTES)
    return fail(RMSMP_EWORKSPACE, "conv2d_static_workspace: this layer needs " + std::to_string(need) +
                                      " bytes of workspace, the static one holds " +
                                      std::to_string((size_t)RMSMP_STATIC_WORKSPACE_BYTES));
  void* ws = nullptr;
  st = static_workspace(&ws);
  if (st != RMSMP_OK) return st;
  return rmsmp_conv2d(Wp, X, d, ep, Y, ws, (size_t)RMSMP_STATIC_WORKSPACE_BYTES, stream);
}

rmsmp_status rmsmp_fake_quant_rows(const float* W, int64_t M, int64_t K, const uint8_t* scheme, const float* alpha,
                                   float* What, float* alpha_out, void* stream) {
  if (M < 0 || K < 0) return fail(RMSMP_ESHAPE, "fake_quant_rows: M, K < 0");
  if (M == 0 || K == 0) return RMSMP_OK;
  if (!W || !scheme || !What) return fail(RMSMP_EINVAL, "fake_quant_rows: NULL W, scheme or What");
  if (M > 0x7fffffff) return fail(RMSMP_ESHAPE, "fake_quant_rows: more than 2^31-1 rows");
  rmsmp::FakeQuantArgs a;
  a.W = W;
  a.scheme = scheme;
  a.alpha = alpha;
  a.What = What;
  a.alpha_out = alpha_out;
  a.M = M;
  a.K = K;
  hipError_t e = (hipError_t)rmsmp::launch_fake_quant_rows(a, stream);
  if (e != hipSuccess) return hip_fail(e, "fake_quant_rows: kernel launch");
  return RMSMP_OK;
}

rmsmp_status rmsmp_ste_backward(const float* W, const float* alpha, const float* dWhat, int64_t M, int64_t K,
                                float* dW, void* stream) {
  if (M < 0 || K < 0) return fail(RMSMP_ESHAPE, "ste_backward: M, K < 0");
  if (M == 0 || K == 0) return RMSMP_OK;
  if (!dWhat || !dW) return fail(RMSMP_EINVAL, "ste_backward: NULL dWhat or dW");
  if (alpha && !W) return fail(RMSMP_EINVAL, "ste_backward: W is needed when alpha is given");
  if (M > 0x7fffffff) return fail(RMSMP_ESHAPE, "ste_backward: more than 2^31-1 rows");
  rmsmp::SteArgs a;
  a.W = W;
  a.alpha = alpha;
  a.dWhat = dWhat;
  a.dW = dW;
  a.M = M;
  a.K = K;
  hipError_t e = (hipError_t)rmsmp::launch_ste_backward(a, stream);
  if (e != hipSuccess) return hip_fail(e, "ste_backward: kernel launch");
  return RMSMP_OK;
}

}  // extern "C"
