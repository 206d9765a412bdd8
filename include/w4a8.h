/*
 * w4a8.h -- C-ABI of the MI355X (gfx950) W4A8 quantized linear layer.
 *
 * The scheme is the inference flow of "Dual Precision Quantization" (arXiv 2505.14638, Sec. 3):
 * weights are stored as 4-bit integer codes with per-group scales, are dequantized to FP8 E4M3 at
 * inference time (Eq. 10 / Eq. 14), activations are quantized to FP8 E4M3 with a static per-tensor
 * scale (Eq. 13), the product runs on the FP8 matrix units with wide (fp32) accumulation, and the
 * output leaves in high precision after rescaling (Eq. 4, Eq. 11).
 *
 * Conventions for every entry point
 *   - returns W4A8_OK (0) or a positive w4a8_status; never throws, exits or prints.
 *   - arguments are validated on the host before anything is enqueued: a non-zero return means
 *     nothing was launched (W4A8_ERR_HIP excepted: a launch was refused by the runtime).
 *   - pointers named *_dev are DEVICE pointers owned by the caller; they must stay valid until the
 *     work enqueued on `stream` has completed.  No entry point allocates, frees or synchronizes.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - notation: M tokens, K input features, N output features; W is [N, K] (one row per output
 *     channel), quantization groups are `group_size` consecutive weights along a row (Sec. 3.1,
 *     App. A.1); group g of row n covers k in [g*group_size, (g+1)*group_size).
 *   - size limits (W4A8_ERR_SHAPE beyond them): M, N, K <= 2^30; N * K <= 2^32 weights and N * K / group_size <= 2^25
 *     groups per matrix; tiled layout: ldx8 < 2^23, ldy < 2^20; canonical layout: M * N <= 2^25 outputs per call.
 *   - the FP8 format is E4M3 with range +-448 (Sec. 2.2, Sec. 4.1): bias 7, no infinities,
 *     S.1111.111 is NaN.  The INT4 codes are signed, in [-8, 7]; group scales are non-negative.
 *     The *_asym entry points take the paper's own storage format instead (Sec. 2.1, Eq. 8-9): unsigned
 *     codes in [0, 15] with a per-group zero-point.
 */
#ifndef W4A8_H
#define W4A8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    W4A8_OK = 0,
    W4A8_ERR_NULL = 1,      /* a required pointer is NULL */
    W4A8_ERR_SHAPE = 2,     /* M, N, K or a leading dimension is out of range */
    W4A8_ERR_GROUP = 3,     /* group_size does not divide K, is odd, or is not supported by the layout */
    W4A8_ERR_DTYPE = 4,     /* unknown w4a8_dtype / w4a8_src value */
    W4A8_ERR_LAYOUT = 5,    /* unknown w4a8_layout value, or shape not supported by that layout */
    W4A8_ERR_ALIGN = 6,     /* a pointer or leading dimension misses the required alignment */
    W4A8_ERR_WORKSPACE = 7, /* workspace smaller than w4a8_linear_workspace_bytes() */
    W4A8_ERR_HIP = 8        /* the HIP runtime refused a launch */
} w4a8_status;

/* Every enumeration below spans the whole int range (the two *_RANGE_* enumerators are no values of their own): a caller
   may hand any int to an entry point, which then answers W4A8_ERR_DTYPE / W4A8_ERR_LAYOUT instead of reading an
   enumeration value its type cannot hold. */
typedef enum { W4A8_F32 = 0, W4A8_BF16 = 1, W4A8_DTYPE_RANGE_LO = -0x7FFFFFFF - 1, W4A8_DTYPE_RANGE_HI = 0x7FFFFFFF } w4a8_dtype;

typedef enum {
    W4A8_SRC_F32_RTN = 0,  /* src = W float32 [N, K]; the library quantizes: symmetric round-to-nearest
                              INT4 (Eq. 1, symmetric case of Sec. 2.1): per (row, group)
                              s = max|W| / 7 (s = 1 for an all-zero group),
                              code = clamp(round_half_even(W / s), -8, 7), both divisions in float32 */
    W4A8_SRC_I8_CODES = 1, /* src = int8 codes [N, K], each in [-8, 7] (only the low nibble is kept), plus
                              float32 scales [N, K/group_size] (their magnitude is used): a pure re-layout, for
                              codes produced by an offline calibrator (Alg. 1) */
    W4A8_SRC_F32_RTN_POW2 = 2, /* as W4A8_SRC_F32_RTN with power-of-two scales (Sec. 2.2): s = the smallest power of
                              two >= max|W| / 7 (so that every code stays in [-7, 7]); for w4a8_linear_pow2 */
    W4A8_SRC_RANGE_LO = -0x7FFFFFFF - 1,
    W4A8_SRC_RANGE_HI = 0x7FFFFFFF
} w4a8_src;

typedef enum {
    /* Row-major, two's-complement nibbles.  packed: byte j of row n = (code[n,2j] & 0xF) | ((code[n,2j+1] & 0xF) << 4), N*K/2 bytes.
       scales: float32 [N, K/group_size] row-major.  Any even K, any even group_size dividing K. */
    W4A8_LAYOUT_CANONICAL = 0,
    /* Tiled for the FP8 matrix unit; needs K % 128 == 0 and group_size % 128 == 0.  Rows are padded with
       code 0 / scale 0 up to Np = ceil(N/16)*16.
       packed (Np*K/2 bytes): tile (t, c) = (n / 16, k / 128) is the 1024 bytes at ((t * (K/128)) + c) * 1024.
       A tile is 64 slots of 16 bytes, slot = 16 * ((k % 128) / 32) + (n % 16).  With p = k % 32, d = p / 8,
       e = p % 8, the code sits in byte 4*d + (e % 4) of its slot: low nibble if e < 4, else high nibble.
       Nibbles are sign-magnitude: bit 3 = sign, bits 0..2 = |code| for codes in [-7, 7]; -8 is the pattern 1000.
       scales (Np*K/group_size floats): element (n, g) at ((n / 16) * (K/group_size) + g) * 16 + (n % 16), stored
       as |scale|, with the sign bit set exactly for the (n, g) whose codes contain -8 (a hint that lets the
       kernels expand nibbles the short way elsewhere; the packed codes alone still determine every weight). */
    W4A8_LAYOUT_TILED = 1,
    W4A8_LAYOUT_RANGE_LO = -0x7FFFFFFF - 1,
    W4A8_LAYOUT_RANGE_HI = 0x7FFFFFFF
} w4a8_layout;

/* Sizes of the buffers w4a8_pack_weights writes, in bytes / in floats; 0 for unsupported arguments. */
size_t w4a8_packed_bytes(int64_t N, int64_t K, w4a8_layout layout);
size_t w4a8_scales_count(int64_t N, int64_t K, int32_t group_size, w4a8_layout layout);

/*
 * Activation FP8 quantization, Eq. 13: x8[m,k] = nearest_E4M3( X[m,k] / s_x ).
 *   x_dev      X, [M, K] with row stride ldx elements, float32 or bf16 (x_dtype)
 *   scale_dev  one float32 on the device: the static per-tensor scale s_x (computed offline, Sec. 3.1)
 *   x8_dev     out, E4M3 bytes [M, K] with row stride ldx8 bytes
 * The quotient is one correctly rounded float32 division, rounded once to the nearest E4M3 value with
 * ties to even; magnitudes beyond 448 (infinities included) saturate to +-448; NaN gives a NaN byte; the
 * sign of zero is kept.  M == 0 is a successful no-op.  ldx >= K, ldx8 >= K.
 */
int w4a8_quantize_act(const void* x_dev, w4a8_dtype x_dtype, int64_t M, int64_t K, int64_t ldx,
                      const float* scale_dev, uint8_t* x8_dev, int64_t ldx8, void* stream);

/*
 * Calibration of the static activation scale (Eq. 13: s_x = max|X| / Z_max over calibration data, offline).
 *   w4a8_act_amax             folds max|X| of one batch, X [M, K] float32 or bf16 with row stride ldx elements, into
 *                             *amax_dev (a float32 the caller has set to 0 before the first batch; NaNs are skipped)
 *   w4a8_act_scale_from_amax  writes *scale_dev = *amax_dev / 448 (one float32 division; 1 when the maximum is 0)
 */
int w4a8_act_amax(const void* x_dev, w4a8_dtype x_dtype, int64_t M, int64_t K, int64_t ldx, float* amax_dev, void* stream);
int w4a8_act_scale_from_amax(const float* amax_dev, float* scale_dev, void* stream);

/*
 * Weight packing (offline with respect to inference; part of the boundary because the packed bytes are
 * compared bit for bit).  Writes w4a8_packed_bytes() bytes to packed_dev and w4a8_scales_count() floats to
 * scales_dev in `layout`.  src_scales_dev is read only for W4A8_SRC_I8_CODES (NULL otherwise).
 * group_size = K gives one scale per output channel.
 */
int w4a8_pack_weights(const void* src_dev, w4a8_src src_kind, const float* src_scales_dev,
                      int64_t N, int64_t K, int32_t group_size, w4a8_layout layout,
                      uint8_t* packed_dev, float* scales_dev, void* stream);

/*
 * Bytes of device scratch with which w4a8_linear runs these sizes fastest (tiled layout); 0 for most shapes.
 * Non-zero where the layer has few output tiles and a deep K (Sec. 1: between the memory-bound and the compute-bound
 * regime -- some 41 to 512 tokens on the down projection of a decoder): K is then multiplied in several ranges by different
 * workgroups, whose float32 partial sums (ranges x M x round_up(N, 64) floats) pass through the scratch and are
 * added in the order of the ranges by a second launch, so the result does not depend on timing.
 */
size_t w4a8_linear_workspace_bytes(int64_t M, int64_t K, int64_t N, int32_t group_size);

/*
 * The quantized linear layer (Sec. 3; Eq. 10, Eq. 4, Eq. 11):
 *   Y[m,n] = cast( s_x * sum_g s_w[n,g] * sum_{k in g} val(x8[m,k]) * code[n,k] )
 * The INT4 codes are expanded in registers to the E4M3 bytes of the same integers (exact: at most four
 * significant bits), multiplied against the E4M3 activations on the FP8 matrix units with fp32
 * accumulation; each group's partial sum is scaled by s_w[n,g] in fp32, the total by s_x.
 *   x8_dev        E4M3 activations [M, K], row stride ldx8 bytes (TILED: ldx8 % 16 == 0, 16-byte aligned)
 *   x_scale_dev   one float32 on the device: s_x
 *   packed_dev, w_scales_dev   as written by w4a8_pack_weights for the same N, K, group_size, layout
 *   y_dev         out [M, N], float32 or bf16 (round to nearest even), row stride ldy elements
 *   workspace_dev NULL: the layer runs without scratch (slower where w4a8_linear_workspace_bytes() is not 0, same
 *                 tolerance).  Not NULL: 16-byte aligned device memory of workspace_bytes bytes, which must be at least
 *                 w4a8_linear_workspace_bytes() for these sizes (W4A8_ERR_WORKSPACE otherwise); its contents are
 *                 scratch, owned by the call until the stream work completes (a launch captured into a HIP graph uses it
 *                 at every replay: it has to outlive the graph).
 * Kernel choice depends only on (M, K, N, layout) and on whether a workspace is given: up to 32 tokens (up to 64 on
 * layers of at most 4096 channels, or of at most 8192 when K >= 8192; up to 48 on at most 6144 channels) take the
 * bandwidth-bound few-token path, larger M the MFMA-tiled paths; with a workspace the shapes
 * w4a8_linear_workspace_bytes() names (from 41 tokens on) run K in ranges across workgroups instead.  CANONICAL always
 * takes a plain reference-speed kernel.  M == 0 is a no-op.
 */
int w4a8_linear(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                const uint8_t* packed_dev, const float* w_scales_dev, int64_t N, int32_t group_size,
                w4a8_layout layout, void* y_dev, w4a8_dtype y_dtype, int64_t ldy,
                void* workspace_dev, size_t workspace_bytes, void* stream);

/*
 * w4a8_linear for callers that cannot allocate device memory (code under HIP graph capture, serving loops, harnesses
 * that forbid it): the same layer, tiled layout, with the scratch of w4a8_linear_workspace_bytes() taken from a buffer
 * of W4A8_STATIC_WORKSPACE_BYTES that lives inside the library (one per GPU, held until the process ends) instead of a
 * workspace argument.  Calls nothing that allocates or frees.  Sizes whose scratch would exceed the buffer return
 * W4A8_ERR_WORKSPACE (use w4a8_linear with a workspace of your own, or with none).  All calls on one GPU share the
 * buffer: two calls whose stream work can overlap in time on the same GPU race on it; calls ordered on one stream do not.
 * Output identical to w4a8_linear with a sufficient workspace.
 */
#define W4A8_STATIC_WORKSPACE_BYTES (16u << 20)
int w4a8_linear_static_workspace(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                                 const uint8_t* packed_dev, const float* w_scales_dev, int64_t N, int32_t group_size,
                                 void* y_dev, w4a8_dtype y_dtype, int64_t ldy, void* stream);

/*
 * w4a8_quantize_act and w4a8_linear in one launch, for few tokens (the memory-bound regime, where a separate
 * quantization kernel costs a launch and a round trip of the activations): Y = w4a8_linear(w4a8_quantize_act(X)).
 * Every workgroup quantizes all of X into on-chip memory while its first weights are on their way, with the same
 * single float32 division and rounding per element (Eq. 13), so the codes, and with them Y, are identical bit for bit
 * to the two calls.  x_dev: float32 or bf16 [M, K], row stride ldx elements, 16-byte aligned, ldx a multiple of 4
 * (float32) or 8 (bf16).  x8_out_dev: NULL, or where the FP8 codes are also written, [M, K] bytes with row stride K,
 * 16-byte aligned.  Tiled layout; 1 <= M <= 16 and M * K <= 65536 (W4A8_ERR_SHAPE otherwise: make the two calls);
 * everything else as in w4a8_linear.
 */
int w4a8_linear_quantize_in(const void* x_dev, w4a8_dtype x_dtype, int64_t M, int64_t K, int64_t ldx,
                            const float* x_scale_dev, const uint8_t* packed_dev, const float* w_scales_dev, int64_t N,
                            int32_t group_size, void* y_dev, w4a8_dtype y_dtype, int64_t ldy, uint8_t* x8_out_dev,
                            void* stream);

/*
 * Test hook for Eq. 10: writes the E4M3 byte the fused kernels feed to the matrix unit for every code,
 * w8[n,k] = nearest_E4M3(code[n,k]), row-major [N, K], using the same device routine as w4a8_linear.
 */
int w4a8_dequant_weights(const uint8_t* packed_dev, int64_t N, int64_t K, w4a8_layout layout,
                         uint8_t* w8_dev, void* stream);

/*
 * The same layer in the paper's two-level reading (Eq. 6-11 taken literally): the group scale s8[n,g] lives in the
 * FP8 domain, the FP8 weight is the product rounded onto the E4M3 grid,
 *   w8[n,k] = nearest_E4M3( float32(code[n,k]) * s8[n, k / group_size] )      (float32 product, ties to even,
 *                                                                              saturating at +-448),
 *   Y[m,n]  = cast( s_x * s_w[n] * sum_k val(x8[m,k]) * val(w8[n,k]) ),
 * with the sum over all of K accumulated in fp32 on the matrix units and one rescale at the end (Eq. 11); s_w is the
 * per-channel (per_channel = 1: N floats) or per-tensor (per_channel = 0: one float) scale of Eq. 6.
 *   packed_dev, w_scales8_dev   W4A8_LAYOUT_TILED buffers as written by w4a8_pack_weights from W4A8_SRC_I8_CODES with
 *                               the FP8-domain group scales as its scales
 * Everything else as in w4a8_linear.  w4a8_dequant_weights_two_level writes the bytes w8 row-major [N, K] with the
 * device routine the kernels use (test hook).
 */
int w4a8_linear_two_level(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                          const uint8_t* packed_dev, const float* w_scales8_dev, const float* w_out_scales_dev,
                          int32_t per_channel, int64_t N, int32_t group_size, void* y_dev, w4a8_dtype y_dtype,
                          int64_t ldy, void* stream);
int w4a8_dequant_weights_two_level(const uint8_t* packed_dev, const float* w_scales8_dev, int64_t N, int64_t K,
                                   int32_t group_size, uint8_t* w8_dev, void* stream);

/*
 * The layer for power-of-two group scales (Sec. 2.2: scaling factors that are powers of two turn scaling into an
 * exponent adjustment).  Same definition and arguments as w4a8_linear with W4A8_LAYOUT_TILED; every group scale must
 * be a power of two 2^e with -127 <= e <= 127: only the exponent field of each float32 scale is read (a mantissa is
 * ignored, i.e. the scale is rounded down to a power of two; a zero scale acts as 2^-127).  The FP8 matrix unit
 * applies 2^e to each 32-deep partial sum itself (block-scaled MFMA with an E8M0 scale per lane), so the sum over all
 * of K stays in the unit's fp32 accumulator and the per-group multiply-adds of w4a8_linear disappear.  Buffers as
 * written by w4a8_pack_weights (W4A8_SRC_F32_RTN_POW2, or W4A8_SRC_I8_CODES with power-of-two scales).
 */
int w4a8_linear_pow2(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                     const uint8_t* packed_dev, const float* w_scales_dev, int64_t N, int32_t group_size, void* y_dev,
                     w4a8_dtype y_dtype, int64_t ldy, void* stream);

/*
 * The asymmetric format (Eq. 1 with q_min = 0, q_max = 15; Eq. 8-9; dequantization by Eq. 14): unsigned 4-bit codes u
 * with a scale s[n,g] and a zero-point z[n,g] per (row, group), z an integer in [0, 15] like the codes;
 *   Y[m,n] = cast( s_x * sum_g s[n,g] * sum_{k in g} val(x8[m,k]) * (u[n,k] - z[n,g]) ).
 * The integers u - z lie in [-15, 15] and are exact in E4M3: the MFMA-tiled kernel expands each nibble to the E4M3
 * byte of u - z (per lane a 16-entry table built from the zero-point); the few-token kernel feeds the exact
 * half-integer u - 7.5 instead and adds (7.5 - z) * sum_k val(x8) per 128 positions, the sum taken on the matrix unit
 * as well.  Both multiply on the FP8 matrix units and apply the group scale to each group's partial sum in fp32, as
 * w4a8_linear does with signed codes.
 * Storage (tiled only; K % 128 == 0, group_size % 128 == 0; rows padded to Np = ceil(N/16)*16 with code 0, scale 0,
 * zero-point 0):
 *   packed  the byte and nibble positions of W4A8_LAYOUT_TILED; the nibble writes the code as u = 7.5 +- (m + 0.5):
 *           bit 3 = 1 for codes 0..7 (then m = 7 - u), bits 0..2 = m (codes 8..15: m = u - 8);
 *   params  w4a8_asym_params_bytes() bytes, 16-byte aligned: one 80-byte record per (16-row band t, group g) at byte
 *           (t * (K/group_size) + g) * 80: the 16 float32 scales of rows 16t .. 16t+15, then their 16 zero-point bytes.
 * w4a8_pack_weights_asym writes both.  src_kind W4A8_SRC_F32_RTN: src = W float32 [N, K]; per (row, group)
 *   lo = min(min W, 0), hi = max(max W, 0), s = (hi - lo) / 15 (1 for an all-zero group), z = round(-lo / s),
 *   u = clamp(round(W / s + z), 0, 15), every step in float32, rounding half to even
 * (the range is made to contain zero so that z fits the 4 bits).  W4A8_SRC_I8_CODES: src = bytes [N, K] holding the
 * codes (only the low nibble is kept), src_scales_dev float32 [N, K/group_size], src_zeros_dev bytes
 * [N, K/group_size] (values above 15 are stored as 15): a pure re-layout for codes from an offline calibrator
 * (Alg. 1).  src_scales_dev and src_zeros_dev are read only for W4A8_SRC_I8_CODES.
 * w4a8_linear_asym: arguments as in w4a8_linear (TILED alignment rules; params_dev in place of the scales), same
 * kernel choice.  w4a8_dequant_weights_asym writes the bytes nearest_E4M3(u - z) row-major [N, K] with the device
 * routine the kernels use (test hook).
 */
size_t w4a8_asym_params_bytes(int64_t N, int64_t K, int32_t group_size);
int w4a8_pack_weights_asym(const void* src_dev, w4a8_src src_kind, const float* src_scales_dev,
                           const uint8_t* src_zeros_dev, int64_t N, int64_t K, int32_t group_size, uint8_t* packed_dev,
                           void* params_dev, void* stream);
int w4a8_linear_asym(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                     const uint8_t* packed_dev, const void* params_dev, int64_t N, int32_t group_size, void* y_dev,
                     w4a8_dtype y_dtype, int64_t ldy, void* stream);
int w4a8_dequant_weights_asym(const uint8_t* packed_dev, const void* params_dev, int64_t N, int64_t K, int32_t group_size,
                              uint8_t* w8_dev, void* stream);

/*
 * The asymmetric format in the two-level reading, i.e. the inference flow exactly as Sec. 3.1 states it (Eq. 8-11):
 * the group scale s8[n,g] and zero-point z[n,g] live in the FP8 domain, the 4-bit code is dequantized to FP8,
 *   w8[n,k] = nearest_E4M3( float32(u[n,k] - z[n,g]) * s8[n,g] )      (one float32 product, ties to even, saturating),
 *   Y[m,n]  = cast( s_x * s_w[n] * sum_k val(x8[m,k]) * val(w8[n,k]) ),
 * with the sum over all of K in fp32 on the matrix units and s_w per channel (per_channel = 1: N floats) or per
 * tensor (per_channel = 0: one float), Eq. 6.  packed_dev and params8_dev are the buffers of w4a8_pack_weights_asym
 * from W4A8_SRC_I8_CODES, with the FP8-domain group scales as its scales (the output of Alg. 1).  Everything else as
 * in w4a8_linear_two_level.  w4a8_dequant_weights_asym_two_level writes the bytes w8 row-major [N, K] (test hook).
 */
int w4a8_linear_asym_two_level(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                               const uint8_t* packed_dev, const void* params8_dev, const float* w_out_scales_dev,
                               int32_t per_channel, int64_t N, int32_t group_size, void* y_dev, w4a8_dtype y_dtype,
                               int64_t ldy, void* stream);
int w4a8_dequant_weights_asym_two_level(const uint8_t* packed_dev, const void* params8_dev, int64_t N, int64_t K,
                                        int32_t group_size, uint8_t* w8_dev, void* stream);

/*
 * Offline calibration (not part of inference; its outputs are the inputs of w4a8_pack_weights_asym with
 * W4A8_SRC_I8_CODES and of w4a8_linear_asym_two_level).
 *
 * w4a8_hessian_accumulate: H += X^T X for one batch of calibration activations (the Hessian of the layer-wise
 * objective, Eq. 5, App. A.2).  x_dev: X [T, K] float32 or bf16, row stride ldx elements; h_dev: float32 [K, K]
 * row-major, in/out (set to 0 before the first batch); float32 accumulation.  K <= 65536.
 *
 * w4a8_hessian_inverse_factor: dampening and Cholesky factorization (Sec. 3.3): from H to the matrix U that
 * w4a8_dpq_calibrate takes.  H_d = P^T H P + damp * mean(diag H) * I, with P the reordering of perm_dev (Sec. 3.2;
 * NULL: none), i.e. H_d[i, j] = H[perm[i], perm[j]] + ...; u_factor_dev receives float32 [K, K] row-major: the
 * upper-triangular U with positive diagonal and H_d^-1 = U^T U, zeros below the diagonal.  Computed in float64 (a
 * Cholesky factorization of the index-reversed H_d and the inverse of its factor; H_d^-1 itself is never formed).
 *   h_dev          float32 [K, K], symmetric (not modified)
 *   damp           the dampening fraction, >= 0 (GPTQ's customary 0.01)
 *   workspace_dev  w4a8_hessian_factor_workspace_bytes(K) bytes, 16-byte aligned
 *   info_dev       out, one int32: 0, or 1 + the index (counted from the END of the reordered columns) of the first
 *                  pivot that was not positive -- H_d is then not positive definite and U holds no usable values
 * K % 128 == 0, K <= 32768.
 *
 * w4a8_gar_permutation: Group-Aware Reordering (Sec. 3.2, App. A.3).  h_diag_dev: the K diagonal entries of the layer's
 * Hessian X^T X.  perm_dev receives K int32: position i of the reordered tensor holds original column perm[i]; columns
 * keep their group, inside a group they are ordered by descending diagonal entry, whole groups by the descending
 * maximum of their entries (ties: lower original index first).  K % 128 == 0, group_size % 128 == 0.
 *
 * w4a8_dpq_calibrate: Dual Precision Quantization, Alg. 1 (Eq. 5-12), for all rows of W.
 *   w_dev         W float32 [N, K] (not modified)
 *   u_factor_dev  float32 [K, K] row-major: U, the upper-triangular Cholesky factor of the inverse (dampened) Hessian
 *                 (H^-1 = U^T U; Sec. 3.3), of the REORDERED columns when perm_dev is given.  Only the upper triangle is read.
 *   w_scale_dev   s_w of Eq. 6: N floats (per_channel = 1) or one (per_channel = 0)
 *   perm_dev      the visiting order of the columns (from w4a8_gar_permutation), or NULL for left to right
 *   codes_dev     out: unsigned 4-bit codes, one per byte, [N, K] in the original column order
 *   scales8_dev   out: float32 [N, K/group_size], the per-group scales of Eq. 8 (FP8 domain), with their original groups
 *   zeros_dev     out: bytes [N, K/group_size], the per-group zero-points of Eq. 8
 *   workspace_dev w4a8_dpq_workspace_bytes(N, K) bytes, 16-byte aligned
 * Per group, at its start (on the group's current weights, the range extended to contain zero):
 *   W8 = val(nearest_E4M3(W / s_w)),  s = (max W8 - min W8) / 15 (1 if that is 0),  z = round(-min W8 / s);
 * per weight, in visiting order: w8 = val(nearest_E4M3(w / s_w)) (Eq. 7); u = clamp(round(w8 / s + z), 0, 15) (Eq. 9);
 * w8_hat = val(nearest_E4M3((u - z) * s)) (Eq. 10, on the grid, as inference computes it); w_hat = w8_hat * s_w
 * (Eq. 11); err = (w - w_hat) / U[q,q]; every later weight w_v of the row becomes w_v - err * U[q,v] (Eq. 12).  Each
 * step is one float32 operation, so the result is reproducible bit for bit.  The search over scales that Sec. 3.3
 * mentions is in w4a8_dpq_calibrate_mse.  K % 128 == 0, group_size % 128 == 0.
 */
int w4a8_hessian_accumulate(const void* x_dev, w4a8_dtype x_dtype, int64_t T, int64_t K, int64_t ldx, float* h_dev,
                            void* stream);
int w4a8_gar_permutation(const float* h_diag_dev, int64_t K, int32_t group_size, int32_t* perm_dev, void* stream);
size_t w4a8_hessian_factor_workspace_bytes(int64_t K);
int w4a8_hessian_inverse_factor(const float* h_dev, int64_t K, double damp, const int32_t* perm_dev, void* workspace_dev,
                                size_t workspace_bytes, float* u_factor_dev, int32_t* info_dev, void* stream);
size_t w4a8_dpq_workspace_bytes(int64_t N, int64_t K);
int w4a8_dpq_calibrate(const float* w_dev, const float* u_factor_dev, const float* w_scale_dev, int32_t per_channel,
                       const int32_t* perm_dev, int64_t N, int64_t K, int32_t group_size, uint8_t* codes_dev,
                       float* scales8_dev, uint8_t* zeros_dev, void* workspace_dev, size_t workspace_bytes, void* stream);
/* w4a8_dpq_calibrate with the per-group scale search of Sec. 3.3 (the paper names the search, not its grid; this is
 * the reading built here).  At the start of a group, candidate i = 0 .. mse_grid - 1 shrinks the range of Eq. 8 to
 * p_i * [min W8, max W8], p_i = 1 - i * (mse_max_shrink / mse_grid) (float32), derives (s, z) from it, and is scored by
 * sum_k (w8_k - w8_hat_k)^2 over the group's current weights -- w8_hat as inference will see it (Eq. 9 with its
 * clipping to [0, 15], then Eq. 10) -- summed in float32 in visiting order; the first candidate with the smallest score
 * gives the group's parameters.  Candidate 0 is Eq. 8 itself; mse_grid <= 1 is w4a8_dpq_calibrate.
 * 0 <= mse_grid <= 1024, 0 <= mse_max_shrink < 1. */
int w4a8_dpq_calibrate_mse(const float* w_dev, const float* u_factor_dev, const float* w_scale_dev, int32_t per_channel,
                           const int32_t* perm_dev, int64_t N, int64_t K, int32_t group_size, int32_t mse_grid,
                           float mse_max_shrink, uint8_t* codes_dev, float* scales8_dev, uint8_t* zeros_dev,
                           void* workspace_dev, size_t workspace_bytes, void* stream);

/*
 * Elementwise step of the decoder-block linear stack (all linear layers of a block are quantized, Sec. 4.1;
 * this joins gate|up to down): h[m,f] = bf16( silu(gate[m,f]) * up[m,f] ) with gate = gu[m, f],
 * up = gu[m, F + f]; gu_dev is bf16 [M, 2F] with row stride ldgu elements, h_dev bf16 [M, F], stride ldh.
 * Computed in fp32: silu(g) = g / (1 + exp(-g)).
 */
int w4a8_silu_mul(const void* gu_dev, int64_t M, int64_t F, int64_t ldgu, void* h_dev, int64_t ldh, void* stream);

/*
 * Fused forms for a stack of quantized layers (all linear layers of a block are quantized, Sec. 4.1, so the tensor
 * between two of them is only ever read by the next layer's activation quantization, Eq. 13).  Both produce, byte
 * for byte, what the unfused sequence produces -- the bf16 tensor is formed in registers, rounded to bf16 and then
 * quantized with the NEXT layer's static scale -- without writing the bf16 tensor or launching the quantize kernel.
 *   w4a8_linear_fp8_out     = w4a8_linear (W4A8_LAYOUT_TILED, bf16 output) followed by w4a8_quantize_act of that
 *                             output with *y_scale_dev; y8_dev receives E4M3 bytes [M, N], row stride ldy8 bytes.
 *                             Arguments otherwise as in w4a8_linear.
 *   w4a8_silu_mul_quantize  = w4a8_silu_mul followed by w4a8_quantize_act of h with *scale_dev; h8_dev receives E4M3
 *                             bytes [M, F], row stride ldh8 bytes.
 *   w4a8_linear_silu_mul_fp8_out = the gate|up layer (N = 2F output channels), w4a8_silu_mul and the quantization of h
 *                             in one kernel: h8_dev receives E4M3 bytes [M, F].  The weight matrix is the gate|up
 *                             matrix with its rows INTERLEAVED in bands of 16: packed row 32p + i is gate row 16p + i,
 *                             packed row 32p + 16 + i is up row 16p + i (i < 16), so that a workgroup holds both halves
 *                             of the channels it finishes; pack that matrix with w4a8_pack_weights (TILED).
 *                             F % 16 == 0.  The gate and up values are rounded to bf16 before SiLU*mul, as the
 *                             unfused sequence does.
 *   w4a8_linear_quantize_in_fp8_out = w4a8_quantize_act of x followed by w4a8_linear_fp8_out, in one kernel: the form of
 *                             w4a8_linear_quantize_in (same limits: M <= 16, M * K <= 65536; same x, x8_out arguments)
 *                             whose output is quantized for the next layer like that of w4a8_linear_fp8_out.
 */
int w4a8_linear_fp8_out(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                        const uint8_t* packed_dev, const float* w_scales_dev, int64_t N, int32_t group_size,
                        const float* y_scale_dev, uint8_t* y8_dev, int64_t ldy8, void* stream);
int w4a8_linear_quantize_in_fp8_out(const void* x_dev, w4a8_dtype x_dtype, int64_t M, int64_t K, int64_t ldx,
                                    const float* x_scale_dev, const uint8_t* packed_dev, const float* w_scales_dev,
                                    int64_t N, int32_t group_size, const float* y_scale_dev, uint8_t* y8_dev, int64_t ldy8,
                                    uint8_t* x8_out_dev, void* stream);
int w4a8_silu_mul_quantize(const void* gu_dev, int64_t M, int64_t F, int64_t ldgu, const float* scale_dev,
                           uint8_t* h8_dev, int64_t ldh8, void* stream);
int w4a8_linear_silu_mul_fp8_out(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                                 const uint8_t* packed_dev, const float* w_scales_dev, int64_t F, int32_t group_size,
                                 const float* h_scale_dev, uint8_t* h8_dev, int64_t ldh8, void* stream);

/* Static, NUL-terminated description of a status value. */
const char* w4a8_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* W4A8_H */
