/*
 * librmsmp -- row-wise mixed-scheme, multi-precision quantized GEMM for AMD MI355X (gfx950).
 *
 * Inference hot path of RMSMP (ICCV'21, arXiv 2111.00153): inside one layer every
 * weight row (= filter, Fig. 1) carries its own quantization scheme and precision --
 * Fixed-point 4-bit, Power-of-Two 4-bit or Fixed-point 8-bit (Section 3.1, 3.2, Fig. 2) --
 * at a ratio that is the same in every layer (Section 3.2), and multiplies 4-bit Fixed
 * activations (Section 3.1: activations are Fixed for all three schemes).
 *
 * Plain C ABI.  No C++ types, no exceptions and no torch types cross this boundary.
 * Pointers are marked HOST or DEVICE.  Every call returns an rmsmp_status and never
 * aborts; rmsmp_last_error() gives a thread-local message for the last failure.
 * Calls that take a `stream` (a hipStream_t passed as void*, NULL = the null stream)
 * only enqueue work: they do not synchronize and do not allocate.
 */
#ifndef RMSMP_H
#define RMSMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  RMSMP_OK = 0,
  RMSMP_EINVAL = 1,       /* NULL pointer, bad enum / flag value, misaligned buffer */
  RMSMP_ESHAPE = 2,       /* sizes that do not fit together */
  RMSMP_ENOMEM = 3,       /* host or device allocation failed */
  RMSMP_EHIP = 4,         /* a HIP runtime call failed; see rmsmp_last_error() */
  RMSMP_EUNSUPPORTED = 5, /* valid request this build has no kernel for */
  RMSMP_EWORKSPACE = 6    /* workspace missing or too small */
} rmsmp_status;

/* Per-row scheme / precision code (the three candidates of Section 3.2, Fig. 2). */
typedef enum { RMSMP_FIXED4 = 0, RMSMP_POT4 = 1, RMSMP_FIXED8 = 2 } rmsmp_scheme;

/* Packed weights of one layer: opaque, owned by the library, lives in device memory. */
typedef struct rmsmp_packed rmsmp_packed;

const char* rmsmp_last_error(void);
const char* rmsmp_version(void);

/*
 * Row counts for a layer-uniform ratio PoT-4 : Fixed-4 : Fixed-8 = A : B : C, A+B+C = 100
 * (Section 4; Section 3.2 fixes C = 5).  Fixed-8 gets round(M*C/100) rows (at least one
 * when C > 0), PoT-4 round(M*A/100), Fixed-4 the remainder.
 * counts (HOST, 3 entries) = {n_fixed4, n_pot4, n_fixed8}, indexed by rmsmp_scheme.
 */
rmsmp_status rmsmp_ratio_counts(int64_t M, int32_t pct_pot4, int32_t pct_fixed4, int32_t pct_fixed8,
                                int64_t counts[3]);

/*
 * Variance-based choice between PoT-4 and Fixed-4 (Alg. 1, else-branch; Section 3.1):
 * rows whose entry in `scheme` is RMSMP_FIXED8 keep it; of the others, the n_pot4 rows
 * with the lowest weight variance become RMSMP_POT4, the rest RMSMP_FIXED4 (ties by
 * row index).  W: HOST fp32 [M][K].  scheme: HOST, M bytes, read and written.
 */
rmsmp_status rmsmp_assign_by_variance(const float* W, int64_t M, int64_t K, int64_t n_pot4,
                                      uint8_t* scheme);

/*
 * Quantize, encode and upload the weights of one layer.
 *
 *   W       HOST fp32 [M][K], row-major; row r is filter r.  For a convolution
 *           K = C*taps and the K index runs (c, kh, kw) -- the usual OIHW filter tensor.
 *   scheme  HOST, M bytes, each an rmsmp_scheme.
 *   alpha   HOST fp32 [M] or NULL.  NULL: alpha_r = max_k |W[r][k]| (an all-zero row
 *           uses 1).  Weights outside [-alpha, alpha] are clipped (Section 3.1.1).
 *   taps    KH*KW for a convolution layer, 1 for a plain GEMM layer.  K % taps == 0.
 *           A convolution layer with at most 4 input channels (K/taps <= 4) and taps a
 *           square number up to 64 is stored for a square KW x KW filter: it can only be
 *           used with rmsmp_conv2d and KH == KW (EUNSUPPORTED otherwise).
 *   in_perm HOST int32 [K/taps] or NULL: the order in which the input channels arrive.
 *           Channel position j of the activation tensor holds original channel in_perm[j]
 *           (use the row permutation of the layer that produced the activations when that
 *           layer wrote 4-bit output in grouped order).  NULL = identity.
 *
 * Row r is projected on its own level set with its own alpha:
 *   Fixed-m (Eq. 1-2): q = round(Q * clip(w/alpha)), Q = 2^(m-1)-1, level alpha*q/Q;
 *   PoT-4   (Eq. 3-4): level 0 or +-alpha*2^-k, k = 0..6, k = -round(log2 |clip(w/alpha)|),
 *                      zero iff |clip| <= 2^-7;  rounding is half-to-even, all in fp32.
 * Rows are grouped by scheme, 4-bit codes are nibble-packed, and the blob is copied to
 * the current device (synchronously).  On success *out owns the device memory; release
 * it with rmsmp_free_packed.  Errors: EINVAL (NULL, bad scheme code, alpha <= 0),
 * ESHAPE (M, K < 1, K % taps), ENOMEM, EHIP.
 */
rmsmp_status rmsmp_pack_weights(const float* W, int64_t M, int64_t K, const uint8_t* scheme,
                                const float* alpha, int32_t taps, const int32_t* in_perm,
                                rmsmp_packed** out);

/*
 * rmsmp_pack_weights with storage options.  flags = 0 is rmsmp_pack_weights.
 *   RMSMP_PACK_POT_AS_INT8  PoT-4 rows are stored decoded, one byte per weight (their level
 *       2^(6-k) or 0, signed), like Fixed-8 rows: the same levels, scales and results bit for
 *       bit, twice the weight bytes for those rows, and no table decode in the K loop.  On
 *       matrix cores a PoT row multiplies at the same rate as any other and only its decode
 *       costs (the opposite of Section 4's FPGA, where PoT rows are the cheap ones), so this
 *       pays for compute-bound layers -- convolutions, GEMMs with many columns -- and costs
 *       bandwidth where the weights are the traffic (N <= 64).
 * Errors: as rmsmp_pack_weights, plus EINVAL for an unknown flag.
 */
#define RMSMP_PACK_POT_AS_INT8 1u
rmsmp_status rmsmp_pack_weights_opt(const float* W, int64_t M, int64_t K, const uint8_t* scheme,
                                    const float* alpha, int32_t taps, const int32_t* in_perm,
                                    uint32_t flags, rmsmp_packed** out);

void rmsmp_free_packed(rmsmp_packed* p);

/*
 * Describe a packed layer.  Any output pointer may be NULL.  The returned arrays are
 * HOST memory borrowed from `p` (valid until rmsmp_free_packed):
 *   counts[3]  rows per scheme {Fixed-4, PoT-4, Fixed-8}
 *   perm       int32 [M]: grouped position g holds original row perm[g].  4-bit requantized
 *              output (out_kind 2) is written in this grouped order.
 *   rowscale   fp32 [M], original row order: level = rowscale * integer
 *              (alpha/7, alpha*2^-6, alpha/127 for Fixed-4, PoT-4, Fixed-8)
 *   rowsum     int32 [M], original row order: sum_k of the integer weights
 */
rmsmp_status rmsmp_packed_info(const rmsmp_packed* p, int64_t* M, int64_t* K, int64_t counts[3],
                               const int32_t** perm, const float** rowscale, const int32_t** rowsum);

/*
 * Test hook: decode the device blob back to the integer weights.
 * wint: HOST int8 [M][K], original row order and original K order; entry = integer level
 * (Fixed-4: -7..7, PoT-4: 0 or +-2^(6-k), Fixed-8: -127..127).  Synchronizes the device.
 */
rmsmp_status rmsmp_unpack_codes(const rmsmp_packed* p, int8_t* wint);

/*
 * Test hook that needs no GPU: runs the host half of rmsmp_pack_weights (quantize, encode,
 * group, lay out the blob) and decodes the blob again on the host.  Outputs (HOST, each may be
 * NULL): wint int8 [M][K] as in rmsmp_unpack_codes; rowscale fp32 [M]; rowsum int32 [M];
 * perm int32 [M] (grouped position -> original row).
 */
rmsmp_status rmsmp_pack_roundtrip_host(const float* W, int64_t M, int64_t K, const uint8_t* scheme,
                                       const float* alpha, int32_t taps, const int32_t* in_perm,
                                       int8_t* wint, float* rowscale, int32_t* rowsum, int32_t* perm);

/*
 * What happens to the int32 accumulator (fused into the GEMM kernel):
 *   a = acc - act_zero_point * rowsum[r]                         (exact)
 *   out_kind 0: Y = a                                              int32
 *   out_kind 1: y = float(a) * (rowscale[r] * act_scale); y += bias[r]; relu -> Y = y   fp32
 *   out_kind 2: q = clamp(round(y * out_inv_scale), 0, 15)          4-bit code, nibble-packed
 *   out_kind 3: g = GELU(y) = y * Phi(y), Phi the standard normal distribution function, taken
 *               in float64 and rounded to fp32 once (relu must be 0);
 *               q = clamp(round(g * out_inv_scale) + out_zero_point, 0, 15)   4-bit code
 *               -- the activation between the two feed-forward projections of a transformer
 *               layer (the BERT-base workload of Section 4.1), handed on in the affine 4-bit
 *               activation format (real value = s_out * (code - out_zero_point)).
 * Every fp32 operation is rounded on its own (no fused multiply-add); round = half-to-even.
 */
typedef struct {
  float act_scale;        /* s_x: real activation = s_x * (code - act_zero_point) */
  int32_t act_zero_point; /* 0..15 for 4-bit codes, -128..127 for 8-bit codes */
  int32_t act_bits;       /* 4: unsigned codes, two per byte; 8: signed int8 codes */
  const float* bias;      /* DEVICE fp32 [M], original row order, or NULL */
  int32_t relu;           /* 0 or 1 */
  int32_t out_kind;       /* 0, 1, 2 or 3 (see above) */
  float out_inv_scale;    /* 1/s_out, used by out_kind 2 and 3; positive and finite for out_kind 3 */
  int32_t out_zero_point; /* 0..15, used by out_kind 3 */
} rmsmp_epilogue;

/*
 * Y = epilogue( W_packed . X ).           (Alg. 1 forward line: out = proj(input) . proj(W))
 *
 *   X  DEVICE, N columns of K codes, each column contiguous ("[N][K]"): act_bits 4 ->
 *      K/2 bytes per column, element k in byte k/2, even k in the low nibble, K even;
 *      act_bits 8 -> K int8 per column.  The K index is the one W was given in.  16-byte aligned.
 *   Y  DEVICE, caller-allocated:
 *        out_kind 0/1: [M][N] row-major, original row order (int32 / fp32)
 *        out_kind 2/3: [N][M/2] bytes; column n, grouped row g in byte g/2 (even g low nibble);
 *                      M must be even.  This is exactly the X layout of a following layer.
 *   stream  hipStream_t as void*.  Asynchronous; no allocation; no workspace needed.
 * Errors: EINVAL, ESHAPE (N < 0, odd K with 4-bit codes, ...), EHIP.  N == 0 is a no-op.
 */
rmsmp_status rmsmp_gemm(const rmsmp_packed* Wp, const void* X, int64_t N, const rmsmp_epilogue* ep,
                        void* Y, void* stream);

/* Geometry of a 2-D convolution.  Output size OH = (H + 2*pad - KH)/stride + 1, same for OW. */
typedef struct {
  int32_t B, C, H, W, KH, KW, stride, pad;
} rmsmp_conv_desc;

/*
 * Convolution lowered to the same GEMM by im2col (Fig. 1: filters of the weight tensor
 * are rows of the weight matrix); the column index is n = (b*OH + oh)*OW + ow.
 *
 *   Wp  packed with K = C*KH*KW and taps = KH*KW.
 *   X   DEVICE activation codes, NHWC: [B][H][W][C] (4-bit: C/2 bytes per pixel, C even).
 *       Pixels outside the image count as real value 0, i.e. code act_zero_point.
 *   Y   out_kind 0/1: [M][B*OH*OW];  out_kind 2/3: [B][OH][OW][M/2] bytes (NHWC, grouped rows).
 *   workspace  DEVICE scratch of at least rmsmp_conv2d_workspace_size() bytes, or NULL when
 *       that size is 0.  Layers whose C is a multiple of 16, and 8-bit layers with at
 *       most 4 input channels (a network's first layer), run without workspace: the
 *       im2col matrix is never materialised.  Other layers materialise it there.
 * Errors: EINVAL, ESHAPE (K mismatch, empty output), EWORKSPACE, EUNSUPPORTED, EHIP.
 */
rmsmp_status rmsmp_conv2d(const rmsmp_packed* Wp, const void* X, const rmsmp_conv_desc* d,
                          const rmsmp_epilogue* ep, void* Y, void* workspace, size_t workspace_bytes,
                          void* stream);

rmsmp_status rmsmp_conv2d_workspace_size(const rmsmp_packed* Wp, const rmsmp_conv_desc* d,
                                         int32_t act_bits, size_t* bytes);

/*
 * Two convolutions that read the same input tensor, enqueued together: layer A then layer B,
 * each exactly as rmsmp_conv2d computes it (Alg. 1 forward line, once per layer).  Meant for
 * the head of a residual stage of the ResNet-18 workload (Section 4.2): the stride-2 3x3
 * convolution and the stride-2 1x1 projection of the shortcut both read the stage's input.
 * When A is a 3x3 layer and B a 1x1 layer with the same 64, 128 or 256 input channels, 4-bit
 * activations, output kinds 0..2 and shapes the LDS-resident kernel takes, the two run as ONE
 * launch whose work-groups share the compute units (the short 1x1 layer runs in the shadow of
 * the 3x3 layer instead of paying a launch of its own); otherwise the library launches A and
 * then B on the stream.  Results are identical either way.
 *
 *   WpA, dA, epA, YA / WpB, dB, epB, YB   as for rmsmp_conv2d; dA and dB must agree in B, C, H, W,
 *        epA and epB in act_scale, act_zero_point and act_bits; YA != YB.
 *   X    DEVICE, the common input (NHWC codes), 16-byte aligned.
 * Asynchronous on `stream`; allocates nothing; no workspace: a layer that would need one
 * (rmsmp_conv2d_workspace_size > 0) is refused with EWORKSPACE.
 * Errors: as rmsmp_conv2d, plus ESHAPE / EINVAL when the two layers disagree on the input.
 */
rmsmp_status rmsmp_conv2d_pair(const rmsmp_packed* WpA, const rmsmp_conv_desc* dA, const rmsmp_epilogue* epA, void* YA,
                               const rmsmp_packed* WpB, const rmsmp_conv_desc* dB, const rmsmp_epilogue* epB, void* YB,
                               const void* X, void* stream);

/*
 * rmsmp_conv2d for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * rmsmp_conv2d, minus the workspace: layers that need one (see rmsmp_conv2d) materialise their
 * im2col matrix in a buffer of RMSMP_STATIC_WORKSPACE_BYTES that is part of the library's device
 * image; every GPU the library runs on holds its own copy until the process ends.  The call
 * allocates and frees nothing and calls no allocating library routine.
 *   - A layer whose rmsmp_conv2d_workspace_size() exceeds RMSMP_STATIC_WORKSPACE_BYTES is
 *     refused with EWORKSPACE and nothing is launched; use rmsmp_conv2d with your own buffer.
 *   - All calls on one GPU share that GPU's buffer, which keeps the last call's contents (every
 *     byte a call reads it has written first, so nothing needs clearing).  Calls that may overlap
 *     on one GPU -- different streams, different threads -- race on it: keep them on one stream.
 * rmsmp_init() looks the buffer's device address up for the current device (once per device is
 * enough; the first rmsmp_conv2d_static_workspace call on a device does it otherwise).
 * Errors: as rmsmp_conv2d, plus EHIP from the address look-up.
 */
#define RMSMP_STATIC_WORKSPACE_BYTES (16u << 20)
rmsmp_status rmsmp_init(void);
rmsmp_status rmsmp_conv2d_static_workspace(const rmsmp_packed* Wp, const void* X,
                                           const rmsmp_conv_desc* d, const rmsmp_epilogue* ep,
                                           void* Y, void* stream);

/*
 * Weight side of one quantization-aware training step (Alg. 1, loop body), on the device.
 *
 * rmsmp_fake_quant_rows -- forward: What = proj_S(W).  Row r is projected on the level set of
 *   scheme[r] with its own scaling factor, exactly as rmsmp_pack_weights does (Eq. 1-4), and
 *   written back in fp32 as rowscale_r * integer level: the value the packed inference path
 *   multiplies with, bit for bit.
 *     W, What    DEVICE fp32 [M][K] row-major (may not overlap)
 *     scheme     DEVICE, M bytes, each an rmsmp_scheme (device data, not checked: a code above
 *                2 is treated as RMSMP_FIXED8)
 *     alpha      DEVICE fp32 [M] or NULL.  NULL: alpha_r = max_k |W[r][k]| (all-zero row: 1)
 *     alpha_out  DEVICE fp32 [M] or NULL: receives the alpha used
 * rmsmp_ste_backward -- backward, the straight-through estimator (Eq. 5): the gradient with
 *   respect to the projected weights is handed to the weights unchanged (rounding has
 *   derivative 1); the clip in front of the rounding has derivative 0 outside
 *   [-alpha, alpha], so dW[r][k] = 0 where |W[r][k]| > alpha[r].
 *     alpha      DEVICE fp32 [M] or NULL.  NULL (alpha was the row maximum): nothing was
 *                clipped, dW = dWhat and W is not read (may be NULL)
 *     W, dWhat, dW  DEVICE fp32 [M][K]
 * Both are asynchronous on `stream`, allocate nothing, and own nothing.
 * Errors: EINVAL (NULL), ESHAPE (negative sizes, M >= 2^31), EHIP.
 */
rmsmp_status rmsmp_fake_quant_rows(const float* W, int64_t M, int64_t K, const uint8_t* scheme,
                                   const float* alpha, float* What, float* alpha_out, void* stream);
rmsmp_status rmsmp_ste_backward(const float* W, const float* alpha, const float* dWhat, int64_t M,
                                int64_t K, float* dW, void* stream);

/*
 * Test hooks for the kernel dispatch (not part of the method; Section 4 of the paper sizes its
 * three PE arrays once per device, here the launch shape is picked per layer).
 *
 * rmsmp_debug_set_wave_split -- how the four waves of a work-group of the LDS-resident kernel
 *   are shared out: pixel_blocks (2 or 4: 64 or 128 output pixels per wave), k_split (waves that
 *   share one output block, each taking every k_split-th K step), side_by_side (output blocks
 *   next to each other), tile_pairs (pairs of weight tiles per work-group);
 *   k_split * side_by_side * tile_pairs = 4.  The request belongs to the calling thread: it
 *   applies to every later launch from that thread where it fits the layer (otherwise the
 *   automatic choice stays); all zero returns to the automatic choice.
 * rmsmp_debug_last_dispatch -- what the calling thread's last rmsmp_gemm / rmsmp_conv2d ran:
 *   out (HOST, 5 entries) = {kernel, pixel_blocks, k_split, side_by_side, tile_pairs} with kernel
 *   0 none, 1 general, 2 skinny (N <= 64), 3 small-channel rows, 4 first layer (3 channels,
 *   stride 2), 5 LDS-resident, 6 LDS-resident with two layers in one launch (rmsmp_conv2d_pair);
 *   the other four are 0 unless kernel == 5.
 * Errors: EINVAL (negative value, NULL).
 */
rmsmp_status rmsmp_debug_set_wave_split(int32_t pixel_blocks, int32_t k_split, int32_t side_by_side,
                                        int32_t tile_pairs);
rmsmp_status rmsmp_debug_last_dispatch(int32_t out[5]);

/*
 * Test hook that needs no GPU: the break points the kernels use for out_kind 3.  As a function
 * of the fp32 pre-activation y the code is piecewise constant: for y >= *y_split it is the
 * largest c with rise[c] <= y; for y < *y_split it is *fall_base plus the number of j < *n_fall
 * with y <= fall[j].  rise, fall: HOST, 16 floats each (-inf / +inf where a code is always /
 * never reached).  Errors: EINVAL.
 */
rmsmp_status rmsmp_debug_gelu_breakpoints(float out_inv_scale, int32_t out_zero_point, float rise[16],
                                          float fall[16], float* y_split, int32_t* fall_base,
                                          int32_t* n_fall);

/*
 * Measurement hook for benchmarks (not part of the method): what the current device sustains
 * with only int8 matrix instructions in flight (TOP/s, 2 ops per multiply-accumulate, operands
 * in registers) and with only a copy kernel (GB/s, bytes read plus bytes written, 1 GiB each
 * way).  Either pointer (HOST) may be NULL.  Allocates and frees 2 GiB of device memory and
 * synchronizes the device: never call it on a hot path.  Errors: EHIP.
 */
rmsmp_status rmsmp_debug_measure_peaks(double* mfma_int8_tops, double* copy_gbs);

#ifdef __cplusplus
}
#endif
#endif /* RMSMP_H */
