// C-ABI front end: argument validation on the host, then dispatch to the kernel launchers.
// Validation never touches the device, so every error path can be exercised without a GPU.
#include "w4a8_internal.hpp"

#include <atomic>

using namespace w4a8;

// Scratch of w4a8_linear_static_workspace: one copy per GPU, inside the library's device image, held until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress; the device address is looked up per device.
static __device__ __align__(256) unsigned char scratch[W4A8_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::atomic<void*> scratch_ptr[MAX_DEVICES];                   // device address of `scratch` on each GPU, once looked up

// The address of `scratch` on the current device (looked up on the first call there; no allocation), or null.
void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    void* p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return nullptr;
        scratch_ptr[dev].store(p, std::memory_order_release);   // two threads racing here store the same address
    }
    return p;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool valid_dtype(int d) { return d == W4A8_F32 || d == W4A8_BF16; }
inline bool valid_layout(int l) { return l == W4A8_LAYOUT_CANONICAL || l == W4A8_LAYOUT_TILED; }
// Few tokens: the skinny kernel streams the weights once with K split across wavefronts.  From 33 tokens on the
// MFMA-tiled kernels (activations staged once per workgroup, nibble expansion shared by several token blocks) are
// faster, except for narrow layers, where the skinny kernel's finer split of K still wins: up to 64 tokens on layers
// of at most 4096 channels and on deep ones (K >= 8192) of at most 8192, up to 48 tokens on up to 6144 channels
// (measured on the Llama-3 layer shapes with the weights coming from HBM).
inline bool takes_skinny_path(int64_t M, int64_t K, int64_t N) {
    return M <= 32 || (M <= 64 && (N <= 4096 || (K >= 8192 && N <= 8192))) || (M <= 48 && N <= 6144);
}
// ... unless the caller brings a workspace and the layer is deep enough (K >= 12288) for K ranges across workgroups,
// which beat the skinny kernel from 41 tokens on (Llama-3-8B down projection at 48 / 64 tokens: 24 / 29 us against 22)
inline bool prefers_split_k(int64_t M, int64_t K, int64_t N) {
    int cfg, ksplit;
    mfma2d_choose_ksplit(M, K, N, cfg, ksplit);
    return ksplit > 1 && M > 40 && K >= 12288;
}
constexpr int64_t DIM_MAX = (int64_t)1 << 30;      // keeps every 32-bit tile / chunk index in range
// One thread per packed byte, 64 per group scale, 64 per output of the canonical layout's layer: these launches stay
// below 2^32 threads for N * K <= 2^32 weights, N * K / group_size <= 2^25 groups and M * N <= 2^25 canonical outputs.
constexpr int64_t WEIGHTS_MAX = (int64_t)1 << 32, GROUPS_MAX = (int64_t)1 << 25, CANONICAL_OUTPUTS_MAX = (int64_t)1 << 25;

int check_nk(int64_t N, int64_t K, int layout) {
    if (!valid_layout(layout)) return W4A8_ERR_LAYOUT;
    if (N < 1 || K < 2 || N > DIM_MAX || K > DIM_MAX || (K & 1)) return W4A8_ERR_SHAPE;
    if (layout == W4A8_LAYOUT_TILED && K % 128 != 0) return W4A8_ERR_LAYOUT;
    if (((N + 15) / 16 * 16) * K > WEIGHTS_MAX) return W4A8_ERR_SHAPE;
    return W4A8_OK;
}

int check_weight_shape(int64_t N, int64_t K, int64_t G, int layout) {
    if (int e = check_nk(N, K, layout)) return e;
    if (G < 2 || (G & 1) || G > K || K % G != 0) return W4A8_ERR_GROUP;
    if (layout == W4A8_LAYOUT_TILED && G % 128 != 0) return W4A8_ERR_GROUP;
    if (((N + 15) / 16 * 16) * (K / G) > GROUPS_MAX) return W4A8_ERR_SHAPE;
    return W4A8_OK;
}

int check_linear(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* xs, const uint8_t* packed,
                 const float* ws, int64_t N, int32_t G, int layout, void* y, int ydt, int64_t ldy) {
    if (M < 0 || M > DIM_MAX) return W4A8_ERR_SHAPE;
    if (int e = check_weight_shape(N, K, G, layout)) return e;
    if (!valid_dtype(ydt) && ydt != YDT_E4M3) return W4A8_ERR_DTYPE;   // callers with a public y_dtype check it first
    if (ldx8 < K || ldy < N) return W4A8_ERR_SHAPE;
    if (layout == W4A8_LAYOUT_CANONICAL && M * N > CANONICAL_OUTPUTS_MAX) return W4A8_ERR_SHAPE;
    if (layout == W4A8_LAYOUT_TILED && (ldx8 >= ((int64_t)1 << 23) || ldy >= ((int64_t)1 << 20))) return W4A8_ERR_SHAPE;
    if (!x8 || !xs || !packed || !ws || !y) return W4A8_ERR_NULL;
    if (layout == W4A8_LAYOUT_TILED) {
        if (!aligned16(x8) || !aligned16(packed) || !aligned16(ws) || (ldx8 & 15)) return W4A8_ERR_ALIGN;
    }
    if (reinterpret_cast<uintptr_t>(y) % (ydt == W4A8_F32 ? 4 : ydt == W4A8_BF16 ? 2 : 1)) return W4A8_ERR_ALIGN;
    return W4A8_OK;
}

}  // namespace

extern "C" {

size_t w4a8_packed_bytes(int64_t N, int64_t K, w4a8_layout layout) {
    if (check_nk(N, K, layout) != W4A8_OK) return 0;
    const int64_t rows = (layout == W4A8_LAYOUT_TILED) ? ((N + 15) / 16) * 16 : N;
    return (size_t)(rows * (K / 2));
}

size_t w4a8_scales_count(int64_t N, int64_t K, int32_t group_size, w4a8_layout layout) {
    if (check_weight_shape(N, K, group_size, layout) != W4A8_OK) return 0;
    const int64_t rows = (layout == W4A8_LAYOUT_TILED) ? ((N + 15) / 16) * 16 : N;
    return (size_t)(rows * (K / group_size));
}

int w4a8_quantize_act(const void* x_dev, w4a8_dtype x_dtype, int64_t M, int64_t K, int64_t ldx,
                      const float* scale_dev, uint8_t* x8_dev, int64_t ldx8, void* stream) {
    if (!valid_dtype(x_dtype)) return W4A8_ERR_DTYPE;
    if (M < 0 || K < 1 || M > DIM_MAX || K > DIM_MAX || ldx < K || ldx8 < K) return W4A8_ERR_SHAPE;
    if (!x_dev || !scale_dev || !x8_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(x_dev) % (x_dtype == W4A8_F32 ? 4 : 2) || reinterpret_cast<uintptr_t>(scale_dev) % 4)
        return W4A8_ERR_ALIGN;
    if (M == 0) return W4A8_OK;
    return launch_quantize_act(x_dev, x_dtype, M, K, ldx, scale_dev, x8_dev, ldx8, static_cast<hipStream_t>(stream));
}

int w4a8_act_amax(const void* x_dev, w4a8_dtype x_dtype, int64_t M, int64_t K, int64_t ldx, float* amax_dev, void* stream) {
    if (!valid_dtype(x_dtype)) return W4A8_ERR_DTYPE;
    if (M < 0 || K < 1 || M > DIM_MAX || K > DIM_MAX || ldx < K) return W4A8_ERR_SHAPE;
    if (!x_dev || !amax_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(x_dev) % (x_dtype == W4A8_F32 ? 4 : 2) || reinterpret_cast<uintptr_t>(amax_dev) % 4)
        return W4A8_ERR_ALIGN;
    if (M == 0) return W4A8_OK;
    return launch_act_amax(x_dev, x_dtype, M, K, ldx, amax_dev, static_cast<hipStream_t>(stream));
}

int w4a8_act_scale_from_amax(const float* amax_dev, float* scale_dev, void* stream) {
    if (!amax_dev || !scale_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(amax_dev) % 4 || reinterpret_cast<uintptr_t>(scale_dev) % 4) return W4A8_ERR_ALIGN;
    return launch_act_scale(amax_dev, scale_dev, static_cast<hipStream_t>(stream));
}

int w4a8_pack_weights(const void* src_dev, w4a8_src src_kind, const float* src_scales_dev, int64_t N, int64_t K,
                      int32_t group_size, w4a8_layout layout, uint8_t* packed_dev, float* scales_dev, void* stream) {
    if (src_kind != W4A8_SRC_F32_RTN && src_kind != W4A8_SRC_I8_CODES && src_kind != W4A8_SRC_F32_RTN_POW2)
        return W4A8_ERR_DTYPE;
    if (int e = check_weight_shape(N, K, group_size, layout)) return e;
    if (!src_dev || !packed_dev || !scales_dev) return W4A8_ERR_NULL;
    if (src_kind == W4A8_SRC_I8_CODES && !src_scales_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(scales_dev) % 4 || (src_kind != W4A8_SRC_I8_CODES && reinterpret_cast<uintptr_t>(src_dev) % 4))
        return W4A8_ERR_ALIGN;
    return launch_pack_weights(src_dev, src_kind, src_scales_dev, N, K, group_size, layout, packed_dev, scales_dev,
                               static_cast<hipStream_t>(stream));
}

size_t w4a8_linear_workspace_bytes(int64_t M, int64_t K, int64_t N, int32_t group_size) {
    if (M < 1 || M > DIM_MAX || check_weight_shape(N, K, group_size, W4A8_LAYOUT_TILED) != W4A8_OK) return 0;
    if (takes_skinny_path(M, K, N) && !prefers_split_k(M, K, N)) return 0;
    int cfg, ksplit;
    mfma2d_choose_ksplit(M, K, N, cfg, ksplit);
    return mfma2d_splitk_bytes(M, N, ksplit);
}

int w4a8_linear(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                const uint8_t* packed_dev, const float* w_scales_dev, int64_t N, int32_t group_size,
                w4a8_layout layout, void* y_dev, w4a8_dtype y_dtype, int64_t ldy, void* workspace_dev,
                size_t workspace_bytes, void* stream) {
    if (!valid_dtype(y_dtype)) return W4A8_ERR_DTYPE;
    if (int e = check_linear(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, layout, y_dev,
                             y_dtype, ldy))
        return e;
    int ksplit = 0, split_cfg = 0;
    if (workspace_dev != nullptr) {
        if (!aligned16(workspace_dev)) return W4A8_ERR_ALIGN;
        const size_t need = layout == W4A8_LAYOUT_TILED ? w4a8_linear_workspace_bytes(M, K, N, group_size) : 0;
        if (workspace_bytes < need) return W4A8_ERR_WORKSPACE;
        if (need > 0) mfma2d_choose_ksplit(M, K, N, split_cfg, ksplit);
    }
    if (M == 0) return W4A8_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (layout == W4A8_LAYOUT_CANONICAL)
        return launch_linear_canonical(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, y_dev,
                                       y_dtype, ldy, st);
    if (takes_skinny_path(M, K, N) && ksplit <= 1)
        return launch_linear_skinny(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, y_dev,
                                    y_dtype, ldy, 0, 0, 0, nullptr, 0, MODE_CODE_EXACT, nullptr, st);
    if (ksplit > 1)                                              // few tiles, deep K: K ranges across workgroups
        return launch_linear_mfma2d(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, y_dev, y_dtype,
                                    ldy, split_cfg, 0, 0, MODE_CODE_EXACT, nullptr, st, ksplit, workspace_dev);
    return launch_linear_mfma_tiled(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, y_dev,
                                    y_dtype, ldy, 0, 0, 0, nullptr, 0, MODE_CODE_EXACT, nullptr, st);
}

int w4a8_linear_static_workspace(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                                 const uint8_t* packed_dev, const float* w_scales_dev, int64_t N, int32_t group_size,
                                 void* y_dev, w4a8_dtype y_dtype, int64_t ldy, void* stream) {
    if (!valid_dtype(y_dtype)) return W4A8_ERR_DTYPE;
    if (int e = check_linear(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, W4A8_LAYOUT_TILED,
                             y_dev, y_dtype, ldy))
        return e;
    const size_t need = w4a8_linear_workspace_bytes(M, K, N, group_size);
    if (need > (size_t)W4A8_STATIC_WORKSPACE_BYTES) return W4A8_ERR_WORKSPACE;
    if (M == 0) return W4A8_OK;
    void* ws = nullptr;
    if (need > 0) {
        ws = static_scratch();
        if (ws == nullptr) return W4A8_ERR_HIP;
    }
    // Nothing in the scratch has to start at zero: every K range writes its whole [M, round_up(N, 64)] plane of partial
    // sums before the second launch reads it, whatever an earlier call left there.
    return w4a8_linear(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, W4A8_LAYOUT_TILED, y_dev,
                       y_dtype, ldy, ws, need, stream);
}

int w4a8_linear_two_level(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                          const uint8_t* packed_dev, const float* w_scales8_dev, const float* w_out_scales_dev,
                          int32_t per_channel, int64_t N, int32_t group_size, void* y_dev, w4a8_dtype y_dtype,
                          int64_t ldy, void* stream) {
    if (!valid_dtype(y_dtype)) return W4A8_ERR_DTYPE;
    if (int e = check_linear(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales8_dev, N, group_size,
                             W4A8_LAYOUT_TILED, y_dev, y_dtype, ldy))
        return e;
    if (!w_out_scales_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(w_out_scales_dev) % 4) return W4A8_ERR_ALIGN;
    if (per_channel != 0 && per_channel != 1) return W4A8_ERR_DTYPE;
    if (M == 0) return W4A8_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (takes_skinny_path(M, K, N))                              // same kernel choice as w4a8_linear
        return launch_linear_skinny(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales8_dev, N, group_size, y_dev,
                                    y_dtype, ldy, 0, 0, 0, w_out_scales_dev, per_channel, MODE_TWO_LEVEL, nullptr, st);
    return launch_linear_mfma_tiled(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales8_dev, N, group_size, y_dev,
                                    y_dtype, ldy, 0, 0, 0, w_out_scales_dev, per_channel, MODE_TWO_LEVEL, nullptr, st);
}

int w4a8_linear_two_level_variant(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                                  const uint8_t* packed_dev, const float* w_scales8_dev, const float* w_out_scales_dev,
                                  int32_t per_channel, int64_t N, int32_t group_size, void* y_dev, w4a8_dtype y_dtype,
                                  int64_t ldy, int32_t tile, int32_t group_m_workgroups, void* stream) {
    if (!valid_dtype(y_dtype)) return W4A8_ERR_DTYPE;
    if (int e = check_linear(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales8_dev, N, group_size,
                             W4A8_LAYOUT_TILED, y_dev, y_dtype, ldy))
        return e;
    if (!w_out_scales_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(w_out_scales_dev) % 4) return W4A8_ERR_ALIGN;
    if (per_channel != 0 && per_channel != 1) return W4A8_ERR_DTYPE;
    if (tile < 0 || group_m_workgroups < 0) return W4A8_ERR_SHAPE;
    if (M == 0) return W4A8_OK;
    return launch_linear_mfma2d(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales8_dev, N, group_size, y_dev, y_dtype,
                                ldy, tile, group_m_workgroups & 0xFF, group_m_workgroups >> 8, MODE_TWO_LEVEL, nullptr,
                                static_cast<hipStream_t>(stream), 1, nullptr, w_out_scales_dev, per_channel);
}

int w4a8_linear_quantize_in(const void* x_dev, w4a8_dtype x_dtype, int64_t M, int64_t K, int64_t ldx,
                            const float* x_scale_dev, const uint8_t* packed_dev, const float* w_scales_dev, int64_t N,
                            int32_t group_size, void* y_dev, w4a8_dtype y_dtype, int64_t ldy, uint8_t* x8_out_dev,
                            void* stream) {
    if (!valid_dtype(x_dtype) || !valid_dtype(y_dtype)) return W4A8_ERR_DTYPE;
    if (M < 0 || M > 16) return W4A8_ERR_SHAPE;
    if (int e = check_weight_shape(N, K, group_size, W4A8_LAYOUT_TILED)) return e;
    if (M * K > 65536 || ldx < K || ldy < N) return W4A8_ERR_SHAPE;
    if (!x_dev || !x_scale_dev || !packed_dev || !w_scales_dev || !y_dev) return W4A8_ERR_NULL;
    if (!aligned16(x_dev) || ldx % (x_dtype == W4A8_F32 ? 4 : 8) != 0 || !aligned16(packed_dev) || !aligned16(w_scales_dev) ||
        !aligned16(x8_out_dev) || reinterpret_cast<uintptr_t>(x_scale_dev) % 4 ||
        reinterpret_cast<uintptr_t>(y_dev) % (y_dtype == W4A8_F32 ? 4 : 2))
        return W4A8_ERR_ALIGN;
    if (M == 0) return W4A8_OK;
    return launch_linear_skinny(static_cast<const uint8_t*>(x_dev), M, K, ldx, x_scale_dev, packed_dev, w_scales_dev, N,
                                group_size, y_dev, y_dtype, ldy, 0, 0, 0, nullptr, 0, MODE_CODE_EXACT, nullptr,
                                static_cast<hipStream_t>(stream), x_dtype == W4A8_F32 ? 1 : 2, x8_out_dev);
}

int w4a8_linear_variant(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                        const uint8_t* packed_dev, const float* w_scales_dev, int64_t N, int32_t group_size,
                        void* y_dev, w4a8_dtype y_dtype, int64_t ldy, int32_t path, int32_t param0, int32_t param1,
                        void* stream) {
    if (!valid_dtype(y_dtype)) return W4A8_ERR_DTYPE;
    if (int e = check_linear(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size,
                             W4A8_LAYOUT_TILED, y_dev, y_dtype, ldy))
        return e;
    if (M == 0) return W4A8_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (path == 0) {
        if (M > 64 || param0 < 0 || param1 < 0 || (param1 & 0xFF) > 16) return W4A8_ERR_SHAPE;
        return launch_linear_skinny(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, y_dev,
                                    y_dtype, ldy, param0, param1 & 0xFF, param1 >> 8, nullptr, 0, MODE_CODE_EXACT, nullptr, st);
    }
    if (path == 1)
        return launch_linear_mfma_tiled(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, y_dev,
                                        y_dtype, ldy, param0, param1 & 0xFF, param1 >> 8, nullptr, 0, MODE_CODE_EXACT, nullptr, st);
    if (path == 2 || path == 2 + 16 * MODE_POW2)
        return launch_linear_mfma2d(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, y_dev, y_dtype,
                                    ldy, param0, param1 & 0xFF, param1 >> 8, path >> 4, nullptr, st);
    return W4A8_ERR_SHAPE;
}

int w4a8_linear_launch_shape(int64_t M, int64_t K, int64_t N, int32_t group_size, int32_t with_workspace, int32_t* shape4) {
    if (!shape4) return W4A8_ERR_NULL;
    if (M < 1 || M > DIM_MAX) return W4A8_ERR_SHAPE;
    if (int e = check_weight_shape(N, K, group_size, W4A8_LAYOUT_TILED)) return e;
    shape4[0] = shape4[1] = shape4[2] = shape4[3] = 0;
    if (takes_skinny_path(M, K, N) && !(with_workspace && prefers_split_k(M, K, N))) {
        int nt = 0, waves = 0, depth = 0;
        if (!skinny_launch_shape(M, K, N, W4A8_BF16, MODE_CODE_EXACT, 0, nt, waves, depth)) return W4A8_ERR_SHAPE;
        shape4[1] = nt;
        shape4[2] = waves | (depth << 8);
        return W4A8_OK;
    }
    int cfg = 0, ksplit = 0;
    if (with_workspace) mfma2d_choose_ksplit(M, K, N, cfg, ksplit);
    if (ksplit > 1) {
        shape4[0] = 3;
        shape4[1] = cfg;
        shape4[3] = ksplit;
        return W4A8_OK;
    }
    int mf = 0, ks = 0, tpw = 0, cfg2d = -1;
    if (!mfma_launch_shape(M, K, N, MODE_CODE_EXACT, mf, ks, tpw, cfg2d)) return W4A8_ERR_SHAPE;
    if (cfg2d >= 0) {
        shape4[0] = 2;
        shape4[1] = cfg2d;
    } else {
        shape4[0] = 1;
        shape4[1] = mf;
        shape4[2] = ks | (tpw << 8);
    }
    return W4A8_OK;
}

int w4a8_linear_few_token_shape(int64_t M, int64_t K, int64_t N, int32_t group_size, int32_t form, int32_t* shape3) {
    if (!shape3) return W4A8_ERR_NULL;
    if (M < 1 || M > 64 || form < 0 || form > 4) return W4A8_ERR_SHAPE;
    if (int e = check_weight_shape(N, K, group_size, W4A8_LAYOUT_TILED)) return e;
    if (form >= 3 && (M > 16 || M * K > 65536)) return W4A8_ERR_SHAPE;
    if (form == 2 && N % 32 != 0) return W4A8_ERR_SHAPE;
    const int ydt = form == 1 || form == 4 ? YDT_E4M3 : form == 2 ? YDT_SILU_E4M3 : (int)W4A8_BF16;
    int nt = 0, waves = 0, depth = 0;
    if (!skinny_launch_shape(M, K, N, ydt, MODE_CODE_EXACT, form >= 3 ? 2 : 0, nt, waves, depth)) return W4A8_ERR_SHAPE;
    shape3[0] = nt;
    shape3[1] = waves;
    shape3[2] = depth;
    return W4A8_OK;
}

int w4a8_linear_splitk_variant(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                               const uint8_t* packed_dev, const float* w_scales_dev, int64_t N, int32_t group_size,
                               void* y_dev, w4a8_dtype y_dtype, int64_t ldy, int32_t tile, int32_t ksplit,
                               void* workspace_dev, size_t workspace_bytes, void* stream) {
    if (!valid_dtype(y_dtype)) return W4A8_ERR_DTYPE;
    if (int e = check_linear(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size,
                             W4A8_LAYOUT_TILED, y_dev, y_dtype, ldy))
        return e;
    if (ksplit < 2 || ksplit > K / 128 || M < 1) return W4A8_ERR_SHAPE;
    if (!workspace_dev) return W4A8_ERR_NULL;
    if (!aligned16(workspace_dev)) return W4A8_ERR_ALIGN;
    if (workspace_bytes < mfma2d_splitk_bytes(M, N, ksplit)) return W4A8_ERR_WORKSPACE;
    return launch_linear_mfma2d(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, y_dev, y_dtype, ldy,
                                tile, 0, 0, MODE_CODE_EXACT, nullptr, static_cast<hipStream_t>(stream), ksplit, workspace_dev);
}

int w4a8_dequant_weights(const uint8_t* packed_dev, int64_t N, int64_t K, w4a8_layout layout, uint8_t* w8_dev,
                         void* stream) {
    if (int e = check_nk(N, K, layout)) return e;
    if (!packed_dev || !w8_dev) return W4A8_ERR_NULL;
    if (layout == W4A8_LAYOUT_TILED && (!aligned16(packed_dev) || !aligned16(w8_dev))) return W4A8_ERR_ALIGN;
    return launch_dequant_weights(packed_dev, N, K, layout, w8_dev, nullptr, nullptr, 0, 0, static_cast<hipStream_t>(stream));
}

int w4a8_dequant_weights_two_level(const uint8_t* packed_dev, const float* w_scales8_dev, int64_t N, int64_t K,
                                   int32_t group_size, uint8_t* w8_dev, void* stream) {
    if (int e = check_weight_shape(N, K, group_size, W4A8_LAYOUT_TILED)) return e;
    if (!packed_dev || !w_scales8_dev || !w8_dev) return W4A8_ERR_NULL;
    if (!aligned16(packed_dev) || !aligned16(w8_dev) || reinterpret_cast<uintptr_t>(w_scales8_dev) % 4) return W4A8_ERR_ALIGN;
    return launch_dequant_weights(packed_dev, N, K, W4A8_LAYOUT_TILED, w8_dev, w_scales8_dev, nullptr, 0, group_size,
                                  static_cast<hipStream_t>(stream));
}

int w4a8_linear_pow2(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                     const uint8_t* packed_dev, const float* w_scales_dev, int64_t N, int32_t group_size, void* y_dev,
                     w4a8_dtype y_dtype, int64_t ldy, void* stream) {
    if (!valid_dtype(y_dtype)) return W4A8_ERR_DTYPE;
    if (int e = check_linear(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, W4A8_LAYOUT_TILED,
                             y_dev, y_dtype, ldy))
        return e;
    if (M == 0) return W4A8_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (takes_skinny_path(M, K, N))                              // same kernel choice as w4a8_linear
        return launch_linear_skinny(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, y_dev,
                                    y_dtype, ldy, 0, 0, 0, nullptr, 0, MODE_POW2, nullptr, st);
    return launch_linear_mfma_tiled(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, y_dev,
                                    y_dtype, ldy, 0, 0, 0, nullptr, 0, MODE_POW2, nullptr, st);
}

int w4a8_linear_fp8_out(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                        const uint8_t* packed_dev, const float* w_scales_dev, int64_t N, int32_t group_size,
                        const float* y_scale_dev, uint8_t* y8_dev, int64_t ldy8, void* stream) {
    if (int e = check_linear(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, W4A8_LAYOUT_TILED,
                             y8_dev, YDT_E4M3, ldy8))
        return e;
    if (!y_scale_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(y_scale_dev) % 4) return W4A8_ERR_ALIGN;
    if (M == 0) return W4A8_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const w4a8_dtype ydt = static_cast<w4a8_dtype>(YDT_E4M3);
    if (takes_skinny_path(M, K, N))                              // same kernel choice as w4a8_linear
        return launch_linear_skinny(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, y8_dev, ydt,
                                    ldy8, 0, 0, 0, nullptr, 0, MODE_CODE_EXACT, y_scale_dev, st);
    return launch_linear_mfma_tiled(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, y8_dev, ydt,
                                    ldy8, 0, 0, 0, nullptr, 0, MODE_CODE_EXACT, y_scale_dev, st);
}

int w4a8_linear_quantize_in_fp8_out(const void* x_dev, w4a8_dtype x_dtype, int64_t M, int64_t K, int64_t ldx,
                                    const float* x_scale_dev, const uint8_t* packed_dev, const float* w_scales_dev,
                                    int64_t N, int32_t group_size, const float* y_scale_dev, uint8_t* y8_dev, int64_t ldy8,
                                    uint8_t* x8_out_dev, void* stream) {
    if (!valid_dtype(x_dtype)) return W4A8_ERR_DTYPE;
    if (M < 0 || M > 16) return W4A8_ERR_SHAPE;
    if (int e = check_weight_shape(N, K, group_size, W4A8_LAYOUT_TILED)) return e;
    if (M * K > 65536 || ldx < K || ldy8 < N) return W4A8_ERR_SHAPE;
    if (!x_dev || !x_scale_dev || !packed_dev || !w_scales_dev || !y_scale_dev || !y8_dev) return W4A8_ERR_NULL;
    if (!aligned16(x_dev) || ldx % (x_dtype == W4A8_F32 ? 4 : 8) != 0 || !aligned16(packed_dev) || !aligned16(w_scales_dev) ||
        !aligned16(x8_out_dev) || reinterpret_cast<uintptr_t>(x_scale_dev) % 4 || reinterpret_cast<uintptr_t>(y_scale_dev) % 4)
        return W4A8_ERR_ALIGN;
    if (M == 0) return W4A8_OK;
    return launch_linear_skinny(static_cast<const uint8_t*>(x_dev), M, K, ldx, x_scale_dev, packed_dev, w_scales_dev, N,
                                group_size, y8_dev, static_cast<w4a8_dtype>(YDT_E4M3), ldy8, 0, 0, 0, nullptr, 0,
                                MODE_CODE_EXACT, y_scale_dev, static_cast<hipStream_t>(stream), x_dtype == W4A8_F32 ? 1 : 2,
                                x8_out_dev);
}

int w4a8_linear_silu_mul_fp8_out(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                                 const uint8_t* packed_dev, const float* w_scales_dev, int64_t F, int32_t group_size,
                                 const float* h_scale_dev, uint8_t* h8_dev, int64_t ldh8, void* stream) {
    if (F < 16 || F > DIM_MAX / 2 || F % 16 != 0) return W4A8_ERR_SHAPE;
    if (ldh8 < F) return W4A8_ERR_SHAPE;
    if (int e = check_linear(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, 2 * F, group_size, W4A8_LAYOUT_TILED,
                             h8_dev, YDT_E4M3, 2 * F))
        return e;
    if (!h_scale_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(h_scale_dev) % 4) return W4A8_ERR_ALIGN;
    if (M == 0) return W4A8_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const w4a8_dtype ydt = static_cast<w4a8_dtype>(YDT_SILU_E4M3);
    const int64_t N = 2 * F;
    if (takes_skinny_path(M, K, N))                              // same kernel choice as w4a8_linear
        return launch_linear_skinny(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, h8_dev, ydt,
                                    ldh8, 0, 0, 0, nullptr, 0, MODE_CODE_EXACT, h_scale_dev, st);
    return launch_linear_mfma_tiled(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, w_scales_dev, N, group_size, h8_dev, ydt,
                                    ldh8, 0, 0, 0, nullptr, 0, MODE_CODE_EXACT, h_scale_dev, st);
}

size_t w4a8_asym_params_bytes(int64_t N, int64_t K, int32_t group_size) {
    if (check_weight_shape(N, K, group_size, W4A8_LAYOUT_TILED) != W4A8_OK) return 0;
    return (size_t)(((N + 15) / 16) * (K / group_size) * 80);
}

int w4a8_pack_weights_asym(const void* src_dev, w4a8_src src_kind, const float* src_scales_dev,
                           const uint8_t* src_zeros_dev, int64_t N, int64_t K, int32_t group_size, uint8_t* packed_dev,
                           void* params_dev, void* stream) {
    if (src_kind != W4A8_SRC_F32_RTN && src_kind != W4A8_SRC_I8_CODES) return W4A8_ERR_DTYPE;   // no power-of-two form
    if (int e = check_weight_shape(N, K, group_size, W4A8_LAYOUT_TILED)) return e;
    if (!src_dev || !packed_dev || !params_dev) return W4A8_ERR_NULL;
    if (src_kind == W4A8_SRC_I8_CODES && (!src_scales_dev || !src_zeros_dev)) return W4A8_ERR_NULL;
    if (!aligned16(params_dev) || (src_kind == W4A8_SRC_F32_RTN && reinterpret_cast<uintptr_t>(src_dev) % 4) ||
        (src_kind == W4A8_SRC_I8_CODES && reinterpret_cast<uintptr_t>(src_scales_dev) % 4))
        return W4A8_ERR_ALIGN;
    return launch_pack_weights_asym(src_dev, src_kind, src_scales_dev, src_zeros_dev, N, K, group_size, packed_dev,
                                    static_cast<uint8_t*>(params_dev), static_cast<hipStream_t>(stream));
}

int w4a8_linear_asym(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                     const uint8_t* packed_dev, const void* params_dev, int64_t N, int32_t group_size, void* y_dev,
                     w4a8_dtype y_dtype, int64_t ldy, void* stream) {
    const float* params = static_cast<const float*>(params_dev);
    if (!valid_dtype(y_dtype)) return W4A8_ERR_DTYPE;
    if (int e = check_linear(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, params, N, group_size, W4A8_LAYOUT_TILED, y_dev,
                             y_dtype, ldy))
        return e;
    if (M == 0) return W4A8_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (takes_skinny_path(M, K, N))                              // same kernel choice as w4a8_linear
        return launch_linear_skinny(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, params, N, group_size, y_dev, y_dtype, ldy,
                                    0, 0, 0, nullptr, 0, MODE_ASYM, nullptr, st);
    return launch_linear_mfma_tiled(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, params, N, group_size, y_dev, y_dtype, ldy,
                                    0, 0, 0, nullptr, 0, MODE_ASYM, nullptr, st);
}

int w4a8_linear_asym_two_level(const uint8_t* x8_dev, int64_t M, int64_t K, int64_t ldx8, const float* x_scale_dev,
                               const uint8_t* packed_dev, const void* params8_dev, const float* w_out_scales_dev,
                               int32_t per_channel, int64_t N, int32_t group_size, void* y_dev, w4a8_dtype y_dtype,
                               int64_t ldy, void* stream) {
    const float* params = static_cast<const float*>(params8_dev);
    if (!valid_dtype(y_dtype)) return W4A8_ERR_DTYPE;
    if (int e = check_linear(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, params, N, group_size, W4A8_LAYOUT_TILED, y_dev,
                             y_dtype, ldy))
        return e;
    if (!w_out_scales_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(w_out_scales_dev) % 4) return W4A8_ERR_ALIGN;
    if (per_channel != 0 && per_channel != 1) return W4A8_ERR_DTYPE;
    if (M == 0) return W4A8_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (takes_skinny_path(M, K, N))                              // same kernel choice as w4a8_linear
        return launch_linear_skinny(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, params, N, group_size, y_dev, y_dtype, ldy,
                                    0, 0, 0, w_out_scales_dev, per_channel, MODE_ASYM_TWO, nullptr, st);
    return launch_linear_mfma_tiled(x8_dev, M, K, ldx8, x_scale_dev, packed_dev, params, N, group_size, y_dev, y_dtype, ldy,
                                    0, 0, 0, w_out_scales_dev, per_channel, MODE_ASYM_TWO, nullptr, st);
}

static int dequant_asym(const uint8_t* packed_dev, const void* params_dev, int64_t N, int64_t K, int32_t group_size,
                        uint8_t* w8_dev, int two_level, void* stream) {
    if (int e = check_weight_shape(N, K, group_size, W4A8_LAYOUT_TILED)) return e;
    if (!packed_dev || !params_dev || !w8_dev) return W4A8_ERR_NULL;
    if (!aligned16(packed_dev) || !aligned16(w8_dev) || !aligned16(params_dev)) return W4A8_ERR_ALIGN;
    return launch_dequant_weights(packed_dev, N, K, W4A8_LAYOUT_TILED, w8_dev, nullptr,
                                  static_cast<const uint8_t*>(params_dev), two_level, group_size,
                                  static_cast<hipStream_t>(stream));
}

int w4a8_dequant_weights_asym(const uint8_t* packed_dev, const void* params_dev, int64_t N, int64_t K, int32_t group_size,
                              uint8_t* w8_dev, void* stream) {
    return dequant_asym(packed_dev, params_dev, N, K, group_size, w8_dev, 0, stream);
}

int w4a8_dequant_weights_asym_two_level(const uint8_t* packed_dev, const void* params8_dev, int64_t N, int64_t K,
                                        int32_t group_size, uint8_t* w8_dev, void* stream) {
    return dequant_asym(packed_dev, params8_dev, N, K, group_size, w8_dev, 1, stream);
}

int w4a8_hessian_accumulate(const void* x_dev, w4a8_dtype x_dtype, int64_t T, int64_t K, int64_t ldx, float* h_dev,
                            void* stream) {
    if (!valid_dtype(x_dtype)) return W4A8_ERR_DTYPE;
    if (T < 0 || K < 1 || T > DIM_MAX || K > 65536 || ldx < K) return W4A8_ERR_SHAPE;
    if (!x_dev || !h_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(x_dev) % (x_dtype == W4A8_F32 ? 4 : 2) || reinterpret_cast<uintptr_t>(h_dev) % 4)
        return W4A8_ERR_ALIGN;
    if (T == 0) return W4A8_OK;
    return launch_hessian_accumulate(x_dev, x_dtype, T, K, ldx, h_dev, static_cast<hipStream_t>(stream));
}

int w4a8_gar_permutation(const float* h_diag_dev, int64_t K, int32_t group_size, int32_t* perm_dev, void* stream) {
    if (int e = check_weight_shape(1, K, group_size, W4A8_LAYOUT_TILED)) return e;
    if (!h_diag_dev || !perm_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(h_diag_dev) % 4 || reinterpret_cast<uintptr_t>(perm_dev) % 4) return W4A8_ERR_ALIGN;
    return launch_gar_permutation(h_diag_dev, K, group_size, perm_dev, static_cast<hipStream_t>(stream));
}

size_t w4a8_hessian_factor_workspace_bytes(int64_t K) {
    if (K < 128 || K % 128 != 0 || K > 32768) return 0;
    return hessian_factor_workspace_bytes(K);
}

int w4a8_hessian_inverse_factor(const float* h_dev, int64_t K, double damp, const int32_t* perm_dev, void* workspace_dev,
                                size_t workspace_bytes, float* u_factor_dev, int32_t* info_dev, void* stream) {
    if (K < 128 || K % 128 != 0 || K > 32768) return W4A8_ERR_SHAPE;
    if (!(damp >= 0.0) || !(damp <= 1.0e6)) return W4A8_ERR_SHAPE;
    if (!h_dev || !workspace_dev || !u_factor_dev || !info_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(h_dev) % 4 || reinterpret_cast<uintptr_t>(u_factor_dev) % 4 ||
        reinterpret_cast<uintptr_t>(perm_dev) % 4 || reinterpret_cast<uintptr_t>(info_dev) % 4 || !aligned16(workspace_dev))
        return W4A8_ERR_ALIGN;
    if (workspace_bytes < w4a8_hessian_factor_workspace_bytes(K)) return W4A8_ERR_WORKSPACE;
    return launch_hessian_inverse_factor(h_dev, K, damp, perm_dev, workspace_dev, u_factor_dev, info_dev,
                                         static_cast<hipStream_t>(stream));
}

size_t w4a8_dpq_workspace_bytes(int64_t N, int64_t K) {
    if (check_nk(N, K, W4A8_LAYOUT_TILED) != W4A8_OK) return 0;
    return (size_t)(N * K + N * 128) * sizeof(float);
}

int w4a8_dpq_calibrate(const float* w_dev, const float* u_factor_dev, const float* w_scale_dev, int32_t per_channel,
                       const int32_t* perm_dev, int64_t N, int64_t K, int32_t group_size, uint8_t* codes_dev,
                       float* scales8_dev, uint8_t* zeros_dev, void* workspace_dev, size_t workspace_bytes, void* stream) {
    return w4a8_dpq_calibrate_mse(w_dev, u_factor_dev, w_scale_dev, per_channel, perm_dev, N, K, group_size, 0, 0.0f,
                                  codes_dev, scales8_dev, zeros_dev, workspace_dev, workspace_bytes, stream);
}

int w4a8_dpq_calibrate_mse(const float* w_dev, const float* u_factor_dev, const float* w_scale_dev, int32_t per_channel,
                           const int32_t* perm_dev, int64_t N, int64_t K, int32_t group_size, int32_t mse_grid,
                           float mse_max_shrink, uint8_t* codes_dev, float* scales8_dev, uint8_t* zeros_dev,
                           void* workspace_dev, size_t workspace_bytes, void* stream) {
    if (int e = check_weight_shape(N, K, group_size, W4A8_LAYOUT_TILED)) return e;
    if (mse_grid < 0 || mse_grid > 1024) return W4A8_ERR_SHAPE;
    if (mse_grid > 1 && !(mse_max_shrink >= 0.0f && mse_max_shrink < 1.0f)) return W4A8_ERR_SHAPE;
    if (per_channel != 0 && per_channel != 1) return W4A8_ERR_DTYPE;
    if (!w_dev || !u_factor_dev || !w_scale_dev || !codes_dev || !scales8_dev || !zeros_dev || !workspace_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(w_dev) % 4 || reinterpret_cast<uintptr_t>(u_factor_dev) % 4 ||
        reinterpret_cast<uintptr_t>(w_scale_dev) % 4 || reinterpret_cast<uintptr_t>(scales8_dev) % 4 ||
        reinterpret_cast<uintptr_t>(perm_dev) % 4 || !aligned16(workspace_dev))
        return W4A8_ERR_ALIGN;
    if (workspace_bytes < w4a8_dpq_workspace_bytes(N, K)) return W4A8_ERR_WORKSPACE;
    return launch_dpq_calibrate(w_dev, u_factor_dev, w_scale_dev, per_channel, perm_dev, N, K, group_size, codes_dev,
                                scales8_dev, zeros_dev, workspace_dev, mse_grid, mse_max_shrink,
                                static_cast<hipStream_t>(stream));
}

int w4a8_silu_mul(const void* gu_dev, int64_t M, int64_t F, int64_t ldgu, void* h_dev, int64_t ldh, void* stream) {
    if (M < 0 || F < 1 || M > DIM_MAX || F > DIM_MAX || ldgu < 2 * F || ldh < F) return W4A8_ERR_SHAPE;
    if (!gu_dev || !h_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(gu_dev) % 2 || reinterpret_cast<uintptr_t>(h_dev) % 2) return W4A8_ERR_ALIGN;
    if (M == 0) return W4A8_OK;
    return launch_silu_mul(gu_dev, M, F, ldgu, h_dev, ldh, nullptr, static_cast<hipStream_t>(stream));
}

int w4a8_silu_mul_quantize(const void* gu_dev, int64_t M, int64_t F, int64_t ldgu, const float* scale_dev,
                           uint8_t* h8_dev, int64_t ldh8, void* stream) {
    if (M < 0 || F < 1 || M > DIM_MAX || F > DIM_MAX || ldgu < 2 * F || ldh8 < F) return W4A8_ERR_SHAPE;
    if (!gu_dev || !h8_dev || !scale_dev) return W4A8_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(gu_dev) % 2 || reinterpret_cast<uintptr_t>(scale_dev) % 4) return W4A8_ERR_ALIGN;
    if (M == 0) return W4A8_OK;
    return launch_silu_mul(gu_dev, M, F, ldgu, h8_dev, ldh8, scale_dev, static_cast<hipStream_t>(stream));
}

const char* w4a8_status_string(int status) {
    switch (status) {
        case W4A8_OK: return "ok";
        case W4A8_ERR_NULL: return "a required pointer is NULL";
        case W4A8_ERR_SHAPE: return "shape or leading dimension out of range";
        case W4A8_ERR_GROUP: return "group size does not divide K or is not supported by the layout";
        case W4A8_ERR_DTYPE: return "unknown data type or source kind";
        case W4A8_ERR_LAYOUT: return "unknown layout, or shape not supported by the layout";
        case W4A8_ERR_ALIGN: return "pointer or leading dimension is not aligned as required";
        case W4A8_ERR_WORKSPACE: return "workspace too small";
        case W4A8_ERR_HIP: return "the HIP runtime refused a launch";
    }
    return "unknown status";
}

}  // extern "C"
