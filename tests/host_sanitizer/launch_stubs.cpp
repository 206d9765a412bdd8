// Host-only stand-ins for the kernel launchers, for the sanitizer build of the C-ABI front end: validation code runs
// for real (under AddressSanitizer and UndefinedBehaviorSanitizer), nothing is ever launched.
#include "../../paper_2505_14638_amd/csrc/w4a8_internal.hpp"

namespace w4a8 {
int launch_quantize_act(const void*, w4a8_dtype, int64_t, int64_t, int64_t, const float*, uint8_t*, int64_t, hipStream_t) { return W4A8_OK; }
int launch_act_amax(const void*, w4a8_dtype, int64_t, int64_t, int64_t, float*, hipStream_t) { return W4A8_OK; }
int launch_act_scale(const float*, float*, hipStream_t) { return W4A8_OK; }
int launch_pack_weights(const void*, w4a8_src, const float*, int64_t, int64_t, int32_t, w4a8_layout, uint8_t*, float*, hipStream_t) { return W4A8_OK; }
int launch_pack_weights_asym(const void*, w4a8_src, const float*, const uint8_t*, int64_t, int64_t, int32_t, uint8_t*, uint8_t*, hipStream_t) { return W4A8_OK; }
int launch_dequant_weights(const uint8_t*, int64_t, int64_t, w4a8_layout, uint8_t*, const float*, const uint8_t*, int, int32_t, hipStream_t) { return W4A8_OK; }
int launch_linear_canonical(const uint8_t*, int64_t, int64_t, int64_t, const float*, const uint8_t*, const float*, int64_t, int32_t, void*, w4a8_dtype, int64_t, hipStream_t) { return W4A8_OK; }
int launch_linear_skinny(const uint8_t*, int64_t, int64_t, int64_t, const float*, const uint8_t*, const float*, int64_t, int32_t, void*, w4a8_dtype, int64_t, int, int, int, const float*, int, int, const float*, hipStream_t, int, uint8_t*) { return W4A8_OK; }
int launch_linear_mfma_tiled(const uint8_t*, int64_t, int64_t, int64_t, const float*, const uint8_t*, const float*, int64_t, int32_t, void*, w4a8_dtype, int64_t, int, int, int, const float*, int, int, const float*, hipStream_t) { return W4A8_OK; }
int launch_hessian_accumulate(const void*, w4a8_dtype, int64_t, int64_t, int64_t, float*, hipStream_t) { return W4A8_OK; }
int launch_gar_permutation(const float*, int64_t, int32_t, int32_t*, hipStream_t) { return W4A8_OK; }
size_t hessian_factor_workspace_bytes(int64_t K) { return (size_t)(2 * K * K + K * 64 + 2) * 8; }
int launch_hessian_inverse_factor(const float*, int64_t, double, const int32_t*, void*, float*, int32_t*, hipStream_t) { return W4A8_OK; }
int launch_dpq_calibrate(const float*, const float*, const float*, int, const int32_t*, int64_t, int64_t, int32_t, uint8_t*, float*, uint8_t*, void*, int, float, hipStream_t) { return W4A8_OK; }
int launch_silu_mul(const void*, int64_t, int64_t, int64_t, void*, int64_t, const float*, hipStream_t) { return W4A8_OK; }
bool skinny_launch_shape(int64_t, int64_t, int64_t, int, int, int, int& nt, int& waves, int& depth) { nt = 1; waves = 8; depth = 2; return true; }
bool mfma_launch_shape(int64_t, int64_t, int64_t, int, int& mf, int& ks, int& tpw, int& cfg2d) { mf = 16; ks = 1; tpw = 1; cfg2d = -1; return true; }
bool mfma2d_tile(int cfg, int& bm, int& bn) { bm = 256; bn = 256; return cfg >= 0 && cfg <= 5; }
int launch_linear_mfma2d(const uint8_t*, int64_t, int64_t, int64_t, const float*, const uint8_t*, const float*, int64_t, int32_t, void*, w4a8_dtype, int64_t, int, int, int, int, const float*, hipStream_t, int, void*, const float*, int) { return W4A8_OK; }
}  // namespace w4a8
