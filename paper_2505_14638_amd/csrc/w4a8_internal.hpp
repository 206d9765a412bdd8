// Host-side declarations shared by the kernel files and the C-ABI front end.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/w4a8.h"
#include "../../include/w4a8_tuning.h"

namespace w4a8 {

inline int hip_status(hipError_t e) { return e == hipSuccess ? W4A8_OK : W4A8_ERR_HIP; }
inline int launch_status() { return hip_status(hipGetLastError()); }

// How the tiled-layout linear kernels read the weights.
//   MODE_CODE_EXACT  signed codes, fp32 group scales applied to the partial sums
//   MODE_TWO_LEVEL   signed codes, `scales` = FP8-domain group scales, output scaled by s_x * w_out[n] (w_out[0] when
//                    per_channel is 0)
//   MODE_ASYM        unsigned codes, `scales` = the 80-byte records of group scales and zero-points
//   MODE_POW2        signed codes, power-of-two group scales applied by the matrix unit (block-scaled MFMA)
//   MODE_ASYM_TWO    unsigned codes and zero-points with FP8-domain group scales in the 80-byte records: the two-level
//                    reading of the asymmetric format; output scaled like MODE_TWO_LEVEL
enum WeightMode { MODE_CODE_EXACT = 0, MODE_TWO_LEVEL = 1, MODE_ASYM = 2, MODE_POW2 = 3, MODE_ASYM_TWO = 4 };

// What the launchers of the tiled-layout linear kernels pass down to a launch: the operands of w4a8_linear after
// validation.
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
    int mode;                        // a WeightMode
    const float* y_scale;            // FP8 output only: the static scale the output is quantized with (Eq. 13)
    int xq = 0;                      // skinny kernel: x8 is the float32 (1) / bf16 (2) activation matrix, quantized in the kernel
    uint8_t* x8_out = nullptr;       // ... and where its codes go as well (row stride K), or null
};

// Output type beyond the public w4a8_dtype values, for the launchers: E4M3 bytes, the bf16 result quantized with the
// next layer's static activation scale (code-exact mode only).
constexpr int YDT_E4M3 = 2;
// The gate|up layer with SiLU*mul and the next quantization folded in (see SiluFp8): y is E4M3 bytes [M, N / 2].
constexpr int YDT_SILU_E4M3 = 3;

int launch_quantize_act(const void* x, w4a8_dtype dt, int64_t M, int64_t K, int64_t ldx, const float* scale,
                        uint8_t* x8, int64_t ldx8, hipStream_t st);
int launch_act_amax(const void* x, w4a8_dtype dt, int64_t M, int64_t K, int64_t ldx, float* amax, hipStream_t st);
int launch_act_scale(const float* amax, float* scale, hipStream_t st);
int launch_pack_weights(const void* src, w4a8_src kind, const float* src_scales, int64_t N, int64_t K, int32_t G,
                        w4a8_layout layout, uint8_t* packed, float* scales, hipStream_t st);
// asymmetric format (tiled storage): src = float32 weights (W4A8_SRC_F32_RTN) or unsigned codes with their scales and
// zero-points; params = the 80-byte records
int launch_pack_weights_asym(const void* src, w4a8_src kind, const float* src_scales, const uint8_t* src_zeros,
                             int64_t N, int64_t K, int32_t G, uint8_t* packed, uint8_t* params, hipStream_t st);
// tiled layout only: scales8 != nullptr: the two-level bytes nearest_E4M3(code * s8[n,g]); asym_params != nullptr: the
// asymmetric format's bytes nearest_E4M3(code - zero_point[n,g]), or with asym_two_level its two-level bytes
// nearest_E4M3((code - zero_point[n,g]) * s8[n,g])
int launch_dequant_weights(const uint8_t* packed, int64_t N, int64_t K, w4a8_layout layout, uint8_t* w8,
                           const float* scales8, const uint8_t* asym_params, int asym_two_level, int32_t G,
                           hipStream_t st);
int launch_linear_canonical(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x,
                            const uint8_t* packed, const float* scales, int64_t N, int32_t G, void* y,
                            w4a8_dtype ydt, int64_t ldy, hipStream_t st);
// nt / waves / depth = 0: chosen from the shape.  mode: a WeightMode; w_out and per_channel count in MODE_TWO_LEVEL.
int launch_linear_skinny(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x,
                         const uint8_t* packed, const float* scales, int64_t N, int32_t G, void* y, w4a8_dtype ydt,
                         int64_t ldy, int nt, int waves, int depth, const float* w_out, int per_channel, int mode,
                         const float* y_scale, hipStream_t st, int xq = 0, uint8_t* x8_out = nullptr);
// The launch shapes the launchers choose by themselves (requested values other than 0 are kept); false: not built.
bool skinny_launch_shape(int64_t M, int64_t K, int64_t N, int ydt, int mode, int xq, int& nt, int& waves, int& depth);
bool mfma_launch_shape(int64_t M, int64_t K, int64_t N, int mode, int& mf, int& ks, int& tpw, int& cfg2d);
// mf = 16-token blocks per workgroup, ks = K-split groups per workgroup, tpw = weight bands per wavefront; 0: chosen
int launch_linear_mfma_tiled(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x,
                             const uint8_t* packed, const float* scales, int64_t N, int32_t G, void* y,
                             w4a8_dtype ydt, int64_t ldy, int mf, int ks, int tpw, const float* w_out, int per_channel,
                             int mode, const float* y_scale, hipStream_t st);
// Second tiling of the many-token kernel (2-D grid of wavefronts, expansion shared through LDS, persistent workgroups).
// cfg: a tile of mfma2d_tile; group_m = token blocks per super-column of the block order (0: chosen); workgroups = size of
// the persistent grid (0: one per compute unit); mode: MODE_CODE_EXACT, MODE_POW2 or MODE_TWO_LEVEL (w_out, per_channel as
// in the first tiling; float32 / bf16 outputs, no split of K); ksplit > 1: K is multiplied in that
// many ranges by different workgroups, their float32 partial sums go through `workspace` (mfma2d_splitk_bytes).
bool mfma2d_tile(int cfg, int& bm, int& bn);

// Row stride (floats) of a K range's partial sums in the workspace, and the bytes `ksplit` ranges take.
inline int64_t mfma2d_splitk_ldw(int64_t N) { return (N + 63) / 64 * 64; }
inline size_t mfma2d_splitk_bytes(int64_t M, int64_t N, int ksplit) {
    return ksplit > 1 ? (size_t)ksplit * (size_t)M * (size_t)mfma2d_splitk_ldw(N) * sizeof(float) : 0;
}

// The split of K this library uses for a layer of many-token shape when the caller provides a workspace: ksplit = 0 means
// none.  Few output tiles and a deep K (the down projection of a decoder block at 64...512 tokens): the tiles are multiplied
// in `ksplit` K ranges by different workgroups, about as many as it takes to give every compute unit one.  Measured on the
// Llama-3 shapes: 29 -> 22 us at 128 tokens on the 8B down projection (K = 14336), 84 -> 57 us on the 70B one (K = 28672);
// at K = 8192 four or more ranges still win (70B O projection at 192 / 256 tokens: 36 / 38 -> 32 / 35 us) and two lose;
// no gain for K = 4096, where the partial sums (written and read once) weigh as much as the weights.
inline void mfma2d_choose_ksplit(int64_t M, int64_t K, int64_t N, int& cfg, int& ksplit) {
    cfg = 3;
    ksplit = 0;
    const int64_t C = K / 128;
    if (M > 512 || K < 8192) return;
    int64_t tiles = ((M + 127) / 128) * ((N + 255) / 256);      // 128 x 256 tiles ...
    if (tiles <= 16) {                                          // ... or 128 x 128 where those are very few
        cfg = 5;
        tiles = ((M + 127) / 128) * ((N + 127) / 128);
    }
    if (tiles > 128) return;
    int64_t s = 256 / tiles;
    if (s > C / 8) s = C / 8;
    if (s < 2 || (K < 12288 && s < 4)) return;                  // K = 8192: two ranges lose, four or more win (measured)
    const int64_t cps = (C + s - 1) / s;
    s = (C + cps - 1) / cps;                                    // no empty range
    ksplit = s < 2 ? 0 : (int)s;
}

int launch_linear_mfma2d(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x, const uint8_t* packed,
                         const float* scales, int64_t N, int32_t G, void* y, w4a8_dtype ydt, int64_t ldy, int cfg,
                         int group_m, int workgroups, int mode, const float* y_scale, hipStream_t st, int ksplit = 1,
                         void* workspace = nullptr, const float* w_out = nullptr, int per_channel = 0);
int launch_hessian_accumulate(const void* x, w4a8_dtype dt, int64_t T, int64_t K, int64_t ldx, float* h, hipStream_t st);
int launch_gar_permutation(const float* hdiag, int64_t K, int32_t G, int32_t* perm, hipStream_t st);
// U = upper Cholesky factor of the inverse dampened (and reordered) Hessian; workspace: hessian_factor_workspace_bytes(K)
size_t hessian_factor_workspace_bytes(int64_t K);
int launch_hessian_inverse_factor(const float* h, int64_t K, double damp, const int32_t* perm, void* workspace, float* u,
                                  int32_t* info, hipStream_t st);
// workspace: (N * K + N * 128) floats
int launch_dpq_calibrate(const float* w, const float* u, const float* s_w, int per_channel, const int32_t* perm,
                         int64_t N, int64_t K, int32_t G, uint8_t* codes, float* scales, uint8_t* zeros, void* workspace,
                         int mse_grid, float mse_max_shrink, hipStream_t st);
// q_scale != nullptr: h is E4M3 bytes, the bf16 result quantized with *q_scale (Eq. 13)
int launch_silu_mul(const void* gu, int64_t M, int64_t F, int64_t ldgu, void* h, int64_t ldh, const float* q_scale,
                    hipStream_t st);

}  // namespace w4a8
