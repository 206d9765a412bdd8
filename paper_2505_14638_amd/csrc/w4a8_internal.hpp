// Host-side declarations shared by the kernel files and the C-ABI front end.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/w4a8.h"

namespace w4a8 {

inline int hip_status(hipError_t e) { return e == hipSuccess ? W4A8_OK : W4A8_ERR_HIP; }
inline int launch_status() { return hip_status(hipGetLastError()); }

// What the launchers of the tiled-layout linear kernels pass down to a launch: the operands of w4a8_linear after
// validation.  w_out != nullptr selects the two-level mode (scales = FP8-domain group scales, output scaled by
// s_x * w_out[n], or s_x * w_out[0] when per_channel is 0).
struct LinearArgs {
    const uint8_t* x8;
    int M;
    int64_t ldx8;
    const float* s_x;
    const uint8_t* packed;
    const float* scales;
    int N, n_tiles, C, cpg, NG;      // channels, 16-row bands, 128-deep chunks, chunks per group, groups per row
    void* y;
    int64_t ldy;
    const float* w_out;
    int per_channel;
};

int launch_quantize_act(const void* x, w4a8_dtype dt, int64_t M, int64_t K, int64_t ldx, const float* scale,
                        uint8_t* x8, int64_t ldx8, hipStream_t st);
int launch_pack_weights(const void* src, w4a8_src kind, const float* src_scales, int64_t N, int64_t K, int32_t G,
                        w4a8_layout layout, uint8_t* packed, float* scales, hipStream_t st);
// scales8 != nullptr (tiled layout only): the two-level bytes nearest_E4M3(code * s8[n,g])
int launch_dequant_weights(const uint8_t* packed, int64_t N, int64_t K, w4a8_layout layout, uint8_t* w8,
                           const float* scales8, int32_t G, hipStream_t st);
int launch_linear_canonical(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x,
                            const uint8_t* packed, const float* scales, int64_t N, int32_t G, void* y,
                            w4a8_dtype ydt, int64_t ldy, hipStream_t st);
// nt / waves / depth = 0: chosen from the shape.  w_out != nullptr: two-level mode (scales are FP8-domain group scales,
// the output is scaled by s_x * w_out[n], or s_x * w_out[0] when per_channel is 0).
int launch_linear_skinny(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x,
                         const uint8_t* packed, const float* scales, int64_t N, int32_t G, void* y, w4a8_dtype ydt,
                         int64_t ldy, int nt, int waves, int depth, const float* w_out, int per_channel, hipStream_t st);
// mf = 16-token blocks per workgroup, ks = K-split groups per workgroup, tpw = weight bands per wavefront; 0: chosen
int launch_linear_mfma_tiled(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x,
                             const uint8_t* packed, const float* scales, int64_t N, int32_t G, void* y,
                             w4a8_dtype ydt, int64_t ldy, int mf, int ks, int tpw, const float* w_out, int per_channel,
                             hipStream_t st);
int launch_silu_mul(const void* gu, int64_t M, int64_t F, int64_t ldgu, void* h, int64_t ldh, hipStream_t st);

}  // namespace w4a8
