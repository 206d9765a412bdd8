/*
 * w4a8_tuning.h -- tuning and measurement entry points of libw4a8.so.  They are not steps of the layer: the calls of
 * the W4A8 linear layer proper are declared in w4a8.h, whose conventions (status codes, device pointers, streams)
 * apply here too.
 */
#ifndef W4A8_TUNING_H
#define W4A8_TUNING_H

#include "w4a8.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Same as w4a8_linear for W4A8_LAYOUT_TILED with the launch shape chosen by the caller; for tuning sweeps.
 *   path    0 = skinny (M <= 64), 1 = MFMA-tiled (first tiling: one weight band per wavefront),
 *           2 = MFMA-tiled, second tiling (2-D grid of wavefronts, persistent workgroups); 2 + 48 = the same through the
 *           block-scaled MFMA (power-of-two group scales, as w4a8_linear_pow2)
 *   param0  skinny: n-tiles (of 16 rows) per wave, 1, 2 or 4.   tiled: 16-token blocks per workgroup, 4, 8 or 16
 *           (the workgroup covers 16 * param0 tokens); 0 = chosen from the shape
 *   param1  skinny: waves per workgroup (K is split across them), 1..16, plus 256 * chunks in flight per wave
 *           (0 auto, 2 or 4).   tiled: K-split groups per workgroup (1, 2 or 4; 0 = chosen) plus 256 * weight bands
 *           per wavefront (1 or 2; 0 = chosen): the workgroup covers 128 * bands / groups channels.  Built shapes
 *           (blocks, groups, bands): (16,1,1) (8,1,1) (8,2,1) (4,1,1) (4,2,1) (4,4,1) (16,1,2)
 *           path 2: param0 = workgroup tile, 0: 512 x 128, 1: 256 x 256, 2: 256 x 128, 3: 128 x 256, 5: 128 x 128 tokens x
 *           channels (eight wavefronts), 4: 256 x 128 with four wavefronts (two workgroups per compute unit);
 *           param1 = token blocks per super-column of the tile order (0 = chosen) plus 256 * workgroups (0 = chosen)
 * Unsupported combinations return W4A8_ERR_SHAPE.
 */
int w4a8_linear_variant(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                        const uint8_t* packed_dev, const float* w_scales_dev, int64_t N, int32_t group_size,
                        void* y_dev, w4a8_dtype y_dtype, int64_t ldy, int32_t path, int32_t param0,
                        int32_t param1, void* stream);

/*
 * w4a8_linear_two_level on the second tiling with the workgroup tile chosen by the caller (tile, group_m_workgroups as
 * param0 and param1 of path 2 above); arguments otherwise as in w4a8_linear_two_level.  For tests and tuning sweeps.
 */
int w4a8_linear_two_level_variant(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                                  const uint8_t* packed_dev, const float* w_scales8_dev, const float* w_out_scales_dev,
                                  int32_t per_channel, int64_t N, int32_t group_size, void* y_dev, w4a8_dtype y_dtype,
                                  int64_t ldy, int32_t tile, int32_t group_m_workgroups, void* stream);

/*
 * The launch shape w4a8_linear chooses by itself for these sizes (tiled layout, bf16 output), in the terms of
 * w4a8_linear_variant: shape4[0] = path (0, 1 or 2; 3 = the second tiling with K ranges across workgroups, taken only
 * when the caller hands w4a8_linear a workspace -- with_workspace != 0), shape4[1] = param0, shape4[2] = param1,
 * shape4[3] = K ranges (path 3, else 0).  shape4 is HOST memory, four int32.  Nothing is launched.
 */
int w4a8_linear_launch_shape(int64_t M, int64_t K, int64_t N, int32_t group_size, int32_t with_workspace, int32_t* shape4);

/*
 * The launch shape of the few-token kernel (path 0 above) for one of the forms that run on it, M <= 64:
 *   form 0 = w4a8_linear (bf16 / float32 output), 1 = w4a8_linear_fp8_out, 2 = w4a8_linear_silu_mul_fp8_out (N = 2F, the
 *   interleaved gate|up matrix), 3 = w4a8_linear_quantize_in, 4 = w4a8_linear_quantize_in_fp8_out.
 * shape3[0] = weight bands per wavefront, shape3[1] = wavefronts per workgroup (the split of K), shape3[2] = chunks in
 * flight per wavefront.  shape3 is HOST memory, three int32.  Nothing is launched.  The fused forms give the bytes of
 * the sequences they replace because shape3[1] is the same for every form of a given (M, K, N); tests hold it to that.
 */
int w4a8_linear_few_token_shape(int64_t M, int64_t K, int64_t N, int32_t group_size, int32_t form, int32_t* shape3);

/*
 * The second tiling with K multiplied in `ksplit` ranges by different workgroups (what w4a8_linear does with a
 * workspace on the shapes w4a8_linear_workspace_bytes() names), tile and split chosen by the caller.  workspace_dev:
 * 16-byte aligned, at least ksplit * M * round_up(N, 64) * 4 bytes (W4A8_ERR_WORKSPACE otherwise).  tile as param0 of
 * path 2 above; 2 <= ksplit <= K / 128.
 */
int w4a8_linear_splitk_variant(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                               const uint8_t* packed_dev, const float* w_scales_dev, int64_t N, int32_t group_size,
                               void* y_dev, w4a8_dtype y_dtype, int64_t ldy, int32_t tile, int32_t ksplit,
                               void* workspace_dev, size_t workspace_bytes, void* stream);

/*
 * Measurement aids (not part of the layer): the two hardware ceilings the kernels are compared with, measured
 * on the device at hand.  Time the calls with events on `stream`.
 *   w4a8_probe_stream_read  loads every 16 bytes of buf_dev[0 .. bytes) once; bytes / time is the achievable HBM
 *                           read bandwidth when `bytes` is far larger than the caches.  sink_dev: 4 bytes, scratch.
 *   w4a8_probe_mfma_e4m3    issues back-to-back 16x16x128 E4M3 MFMAs on independent accumulators from two
 *                           workgroups per compute unit; w4a8_probe_mfma_flop(iters) / time is the achievable dense
 *                           FP8 MFMA rate.  sink_dev: 4 bytes, scratch.  1 <= iters <= 2^20.
 */
int w4a8_probe_stream_read(const void* buf_dev, size_t bytes, uint32_t* sink_dev, void* stream);
int w4a8_probe_mfma_e4m3(int32_t iters, float* sink_dev, void* stream);
double w4a8_probe_mfma_flop(int32_t iters);

#ifdef __cplusplus
}
#endif
#endif /* W4A8_TUNING_H */
