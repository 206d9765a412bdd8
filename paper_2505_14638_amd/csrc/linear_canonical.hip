// W4A8 linear layer on the canonical (row-major) storage: a plain kernel, one wavefront per output element,
// no matrix unit.  It serves shapes and group sizes the tiled format does not cover and is a second,
// independent device implementation of Eq. 10 / Eq. 4 / Eq. 11 (software E4M3 decode, scalar FMAs).
#include "w4a8_device.hpp"
#include "w4a8_internal.hpp"

namespace w4a8 {
namespace {

// exact value of an E4M3 byte: bias 7, subnormals m * 2^-9, S.1111.111 = NaN
__device__ __forceinline__ float e4m3_value(uint32_t b) {
    const uint32_t e = (b >> 3) & 0xFu, m = b & 7u;
    float v = (e == 0) ? ldexpf((float)m, -9) : ldexpf((float)(8u + m), (int)e - 10);
    if ((b & 0x7Fu) == 0x7Fu) v = __uint_as_float(0x7FC00000u);
    return (b & 0x80u) ? -v : v;
}

template <typename OutT>
__global__ void __launch_bounds__(256) linear_canonical_kernel(const uint8_t* __restrict__ x8, int64_t M, int64_t K,
                                                               int64_t ldx8, const float* __restrict__ s_x,
                                                               const uint8_t* __restrict__ packed,
                                                               const float* __restrict__ scales, int64_t N, int32_t G,
                                                               OutT* __restrict__ y, int64_t ldy) {
    const int64_t wid = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (wid >= M * N) return;
    const int64_t m = wid / N, n = wid - m * N;
    const uint8_t* xr = x8 + m * ldx8;
    const uint8_t* wr = packed + n * (K >> 1);
    const float* sr = scales + n * (K / G);
    float acc = 0.0f;
    for (int64_t j = lane; j < (K >> 1); j += 64) {
        const uint32_t b = wr[j];
        const int q0 = (int)((b & 0xFu) ^ 8u) - 8, q1 = (int)((b >> 4) ^ 8u) - 8;      // sign-extend the nibbles
        const int64_t k = 2 * j;
        acc = fmaf(sr[k / G] * (float)q0, e4m3_value(xr[k]), acc);
        acc = fmaf(sr[(k + 1) / G] * (float)q1, e4m3_value(xr[k + 1]), acc);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) y[m * ldy + n] = OutCast<OutT>::cast(*s_x * acc, 1.0f);
}

}  // namespace

int launch_linear_canonical(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x,
                            const uint8_t* packed, const float* scales, int64_t N, int32_t G, void* y,
                            w4a8_dtype ydt, int64_t ldy, hipStream_t st) {
    const int64_t waves = M * N;
    const unsigned blocks = (unsigned)((waves + 3) / 4);
    if (ydt == W4A8_F32)
        hipLaunchKernelGGL(linear_canonical_kernel<float>, dim3(blocks), dim3(256), 0, st, x8, M, K, ldx8, s_x, packed,
                           scales, N, G, static_cast<float*>(y), ldy);
    else
        hipLaunchKernelGGL(linear_canonical_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st, x8, M, K, ldx8, s_x,
                           packed, scales, N, G, static_cast<uint16_t*>(y), ldy);
    return launch_status();
}

}  // namespace w4a8
