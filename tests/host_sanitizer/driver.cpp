// Drives the argument validation of every entry point of the C-ABI front end (api.hip built for the host with
// AddressSanitizer and UndefinedBehaviorSanitizer, kernel launchers replaced by stubs): the sanitizers abort on the
// first finding; a wrong status prints the line and exits with 1.  No GPU is touched.
#include <cstdint>
#include <cstdio>
#include <cstdlib>

#include "../../include/w4a8.h"
#include "../../include/w4a8_tuning.h"

static int failures = 0;
#define EXPECT(call, want)                                                              \
    do {                                                                                \
        const long long got = (long long)(call);                                        \
        if (got != (long long)(want)) {                                                 \
            std::printf("line %d: %s = %lld, expected %lld\n", __LINE__, #call, got, (long long)(want)); \
            ++failures;                                                                 \
        }                                                                               \
    } while (0)

int main() {
    // a 16-byte aligned address that is never dereferenced on the host: validation looks at values and alignment only
    alignas(256) static unsigned char arena[4096];
    void* P = arena;
    void* P4 = arena + 4;
    const int64_t big = (int64_t)1 << 30;

    EXPECT(w4a8_packed_bytes(1024, 1024, W4A8_LAYOUT_TILED), 1024 * 512);
    EXPECT(w4a8_packed_bytes(17, 128, W4A8_LAYOUT_TILED), 32 * 64);
    EXPECT(w4a8_packed_bytes(big, big, W4A8_LAYOUT_TILED), 0);
    EXPECT(w4a8_scales_count(1024, 1024, 128, W4A8_LAYOUT_TILED), 1024 * 8);
    EXPECT(w4a8_scales_count(big, big, 2, W4A8_LAYOUT_CANONICAL), 0);

    EXPECT(w4a8_quantize_act(P, W4A8_F32, 4, 256, 256, (const float*)P, (uint8_t*)P, 256, nullptr), W4A8_OK);
    EXPECT(w4a8_quantize_act(nullptr, W4A8_F32, 4, 256, 256, (const float*)P, (uint8_t*)P, 256, nullptr), W4A8_ERR_NULL);
    EXPECT(w4a8_quantize_act(P, (w4a8_dtype)7, 4, 256, 256, (const float*)P, (uint8_t*)P, 256, nullptr), W4A8_ERR_DTYPE);
    EXPECT(w4a8_quantize_act(P, W4A8_F32, big + 1, big, big, (const float*)P, (uint8_t*)P, big, nullptr), W4A8_ERR_SHAPE);
    EXPECT(w4a8_quantize_act(arena + 2, W4A8_F32, 4, 256, 256, (const float*)P, (uint8_t*)P, 256, nullptr), W4A8_ERR_ALIGN);

    EXPECT(w4a8_pack_weights(P, W4A8_SRC_F32_RTN, nullptr, 64, 256, 128, W4A8_LAYOUT_TILED, (uint8_t*)P, (float*)P, nullptr), W4A8_OK);
    EXPECT(w4a8_pack_weights(P, W4A8_SRC_I8_CODES, nullptr, 64, 256, 128, W4A8_LAYOUT_TILED, (uint8_t*)P, (float*)P, nullptr), W4A8_ERR_NULL);
    EXPECT(w4a8_pack_weights(P, W4A8_SRC_F32_RTN, nullptr, 64, 256, 96, W4A8_LAYOUT_TILED, (uint8_t*)P, (float*)P, nullptr), W4A8_ERR_GROUP);
    EXPECT(w4a8_pack_weights(P, W4A8_SRC_F32_RTN, nullptr, big, big, 128, W4A8_LAYOUT_TILED, (uint8_t*)P, (float*)P, nullptr), W4A8_ERR_SHAPE);

    auto lin = [&](int64_t M, int64_t K, int64_t ldx8, int64_t N, int32_t G, w4a8_layout layout, int64_t ldy, void* ws, size_t nb) {
        return w4a8_linear((const uint8_t*)P, M, K, ldx8, (const float*)P, (const uint8_t*)P, (const float*)P, N, G, layout, P,
                           W4A8_BF16, ldy, ws, nb, nullptr);
    };
    EXPECT(lin(4, 256, 256, 64, 128, W4A8_LAYOUT_TILED, 64, nullptr, 0), W4A8_OK);
    EXPECT(lin(0, 256, 256, 64, 128, W4A8_LAYOUT_TILED, 64, nullptr, 0), W4A8_OK);
    EXPECT(lin(-1, 256, 256, 64, 128, W4A8_LAYOUT_TILED, 64, nullptr, 0), W4A8_ERR_SHAPE);
    EXPECT(lin(4, 256, 128, 64, 128, W4A8_LAYOUT_TILED, 64, nullptr, 0), W4A8_ERR_SHAPE);
    EXPECT(lin(4, 256, 256, 64, 64, W4A8_LAYOUT_TILED, 64, nullptr, 0), W4A8_ERR_GROUP);
    EXPECT(lin(4, 192, 192, 64, 192, W4A8_LAYOUT_TILED, 64, nullptr, 0), W4A8_ERR_LAYOUT);
    EXPECT(lin(big, big, big, big, 128, W4A8_LAYOUT_TILED, big, nullptr, 0), W4A8_ERR_SHAPE);   // products far beyond 2^32: no overflow
    EXPECT(lin(1 << 13, 64, 64, 1 << 13, 32, W4A8_LAYOUT_CANONICAL, 1 << 13, nullptr, 0), W4A8_ERR_SHAPE);
    const size_t need = w4a8_linear_workspace_bytes(128, 14336, 4096, 128);
    EXPECT(need > 0, 1);
    EXPECT(w4a8_linear_workspace_bytes(128, 4096, 4096, 128), 0);
    EXPECT(w4a8_linear_workspace_bytes(big, big, big, 128), 0);
    EXPECT(lin(128, 14336, 14336, 4096, 128, W4A8_LAYOUT_TILED, 4096, P, need), W4A8_OK);
    EXPECT(lin(128, 14336, 14336, 4096, 128, W4A8_LAYOUT_TILED, 4096, P, need - 1), W4A8_ERR_WORKSPACE);
    EXPECT(lin(128, 14336, 14336, 4096, 128, W4A8_LAYOUT_TILED, 4096, P4, need), W4A8_ERR_ALIGN);
    EXPECT(w4a8_linear_static_workspace((const uint8_t*)P, 512, 28672, 28672, (const float*)P, (const uint8_t*)P, (const float*)P,
                                        8192, 128, P, W4A8_BF16, 8192, nullptr), W4A8_ERR_WORKSPACE);
    EXPECT(w4a8_linear_static_workspace((const uint8_t*)P, 8, 1024, 1024, (const float*)P, (const uint8_t*)P, (const float*)P,
                                        256, 128, P, W4A8_BF16, 256, nullptr), W4A8_OK);
    EXPECT(w4a8_linear_splitk_variant((const uint8_t*)P, 128, 14336, 14336, (const float*)P, (const uint8_t*)P, (const float*)P, 4096,
                                      128, P, W4A8_BF16, 4096, 5, 4, P, (size_t)4 * 128 * 4096 * 4 - 1, nullptr), W4A8_ERR_WORKSPACE);
    int32_t shape[4] = {9, 9, 9, 9};
    EXPECT(w4a8_linear_launch_shape(128, 14336, 4096, 128, 1, shape), W4A8_OK);
    EXPECT(shape[0], 3);
    EXPECT(w4a8_linear_launch_shape(128, 14336, 4096, 128, 1, nullptr), W4A8_ERR_NULL);
    EXPECT(w4a8_linear_launch_shape(128, 14336, 4096, 100, 1, shape), W4A8_ERR_GROUP);
    EXPECT(w4a8_linear_variant((const uint8_t*)P, 100, 256, 256, (const float*)P, (const uint8_t*)P, (const float*)P, 64, 128, P,
                               W4A8_BF16, 64, 0, 1, 1, nullptr), W4A8_ERR_SHAPE);
    EXPECT(w4a8_linear_quantize_in(P, W4A8_BF16, 17, 256, 256, (const float*)P, (const uint8_t*)P, (const float*)P, 64, 128, P,
                                   W4A8_BF16, 64, nullptr, nullptr), W4A8_ERR_SHAPE);
    EXPECT(w4a8_linear_two_level((const uint8_t*)P, 4, 256, 256, (const float*)P, (const uint8_t*)P, (const float*)P, nullptr, 0, 64,
                                 128, P, W4A8_BF16, 64, nullptr), W4A8_ERR_NULL);
    EXPECT(w4a8_linear_pow2((const uint8_t*)P, 4, 256, 256, (const float*)P, (const uint8_t*)P, (const float*)P, 64, 128, P, W4A8_BF16,
                            64, nullptr), W4A8_OK);
    EXPECT(w4a8_linear_asym((const uint8_t*)P, 4, 256, 256, (const float*)P, (const uint8_t*)P, P, 64, 128, P, W4A8_BF16, 64, nullptr),
           W4A8_OK);
    EXPECT(w4a8_linear_fp8_out((const uint8_t*)P, 4, 256, 256, (const float*)P, (const uint8_t*)P, (const float*)P, 64, 128, nullptr,
                               (uint8_t*)P, 64, nullptr), W4A8_ERR_NULL);
    EXPECT(w4a8_linear_silu_mul_fp8_out((const uint8_t*)P, 4, 256, 256, (const float*)P, (const uint8_t*)P, (const float*)P, 24, 128,
                                        (const float*)P, (uint8_t*)P, 24, nullptr), W4A8_ERR_SHAPE);
    EXPECT(w4a8_dequant_weights((const uint8_t*)P, 64, 256, W4A8_LAYOUT_TILED, (uint8_t*)P, nullptr), W4A8_OK);
    EXPECT(w4a8_asym_params_bytes(64, 256, 128), 4 * 2 * 80);
    EXPECT(w4a8_hessian_factor_workspace_bytes(200), 0);
    EXPECT(w4a8_hessian_inverse_factor((const float*)P, 256, 0.01, nullptr, P, 16, (float*)P, (int32_t*)P, nullptr), W4A8_ERR_WORKSPACE);
    EXPECT(w4a8_dpq_workspace_bytes(64, 256), (size_t)(64 * 256 + 64 * 128) * 4);
    EXPECT(w4a8_dpq_calibrate((const float*)P, (const float*)P, (const float*)P, 1, nullptr, 64, 256, 128, (uint8_t*)P, (float*)P,
                              (uint8_t*)P, P, 16, nullptr), W4A8_ERR_WORKSPACE);
    EXPECT(w4a8_silu_mul(P, 4, 64, 64, P, 64, nullptr), W4A8_ERR_SHAPE);
    EXPECT(w4a8_status_string(W4A8_ERR_WORKSPACE) != nullptr, 1);
    if (failures == 0) std::printf("sanitizer driver: all checks passed\n");
    return failures == 0 ? 0 : 1;
}
