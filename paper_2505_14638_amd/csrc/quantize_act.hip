// Activation FP8 quantization (Eq. 13): x8 = nearest_E4M3(X / s_x), static per-tensor s_x.
// Streaming kernel: HBM-bound, 16 elements per thread (one 16-byte store, 128-bit loads).
#include "w4a8_device.hpp"
#include "w4a8_internal.hpp"

namespace w4a8 {
namespace {

template <typename InT>
__global__ void __launch_bounds__(256) quantize_act_vec_kernel(const InT* __restrict__ x, int64_t M, int64_t K16,
                                                               int64_t ldx, const float* __restrict__ scale,
                                                               uint8_t* __restrict__ x8, int64_t ldx8) {
    const float s = *scale;
    const int64_t total = M * K16;
    for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < total; u += (int64_t)gridDim.x * blockDim.x) {
        const int64_t m = u / K16, k = (u - m * K16) * 16;
        float v[16];
        Load16<InT>::load(x + m * ldx + k, v);
        uint4 o;
        o.x = quant4(v[0], v[1], v[2], v[3], s);
        o.y = quant4(v[4], v[5], v[6], v[7], s);
        o.z = quant4(v[8], v[9], v[10], v[11], s);
        o.w = quant4(v[12], v[13], v[14], v[15], s);
        *reinterpret_cast<uint4*>(x8 + m * ldx8 + k) = o;
    }
}

template <typename InT>
__global__ void __launch_bounds__(256) quantize_act_scalar_kernel(const InT* __restrict__ x, int64_t M, int64_t K,
                                                                  int64_t ldx, const float* __restrict__ scale,
                                                                  uint8_t* __restrict__ x8, int64_t ldx8) {
    const float s = *scale;
    const int64_t total = M * K;
    for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < total; u += (int64_t)gridDim.x * blockDim.x) {
        const int64_t m = u / K, k = u - m * K;
        const float t = Load16<InT>::one(x + m * ldx + k) / s;
        x8[m * ldx8 + k] = (uint8_t)(cvt2(t, 0.0f, 0u, false) & 0xFFu);
    }
}

// Static-scale calibration (Eq. 13, offline): running maximum of |X| over calibration batches.  Non-negative floats
// order like their bit patterns, so the maximum is an unsigned integer atomic on the bits; NaNs are skipped.
template <typename InT>
__global__ void __launch_bounds__(256) act_amax_kernel(const InT* __restrict__ x, int64_t M, int64_t K, int64_t ldx,
                                                       uint32_t* __restrict__ amax_bits) {
    float m = 0.0f;
    const int64_t total = M * K;
    for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < total; u += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = u / K, c = u - r * K;
        const float v = fabsf(Load16<InT>::one(x + r * ldx + c));
        m = (v > m) ? v : m;                                     // false for NaN
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if ((threadIdx.x & 63) == 0) atomicMax(amax_bits, __float_as_uint(m));
}

// s_x = amax / 448 as one float32 division (1 when amax is 0, so that the quantizer never divides by zero)
__global__ void act_scale_kernel(const float* __restrict__ amax, float* __restrict__ scale) {
    if (threadIdx.x == 0 && blockIdx.x == 0) scale[0] = (amax[0] == 0.0f) ? 1.0f : __fdiv_rn(amax[0], 448.0f);
}

template <typename InT>
int launch_t(const InT* x, int64_t M, int64_t K, int64_t ldx, const float* scale, uint8_t* x8, int64_t ldx8,
             hipStream_t st) {
    const bool vec = (K % 16 == 0) && (ldx % 16 == 0) && (ldx8 % 16 == 0) &&
                     (reinterpret_cast<uintptr_t>(x) % 16 == 0) && (reinterpret_cast<uintptr_t>(x8) % 16 == 0);
    const int64_t units = vec ? M * (K / 16) : M * K;
    int64_t blocks = (units + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;     // grid-stride beyond 32 workgroups per compute unit
    if (vec)
        hipLaunchKernelGGL(quantize_act_vec_kernel<InT>, dim3((unsigned)blocks), dim3(256), 0, st, x, M, K / 16, ldx,
                           scale, x8, ldx8);
    else
        hipLaunchKernelGGL(quantize_act_scalar_kernel<InT>, dim3((unsigned)blocks), dim3(256), 0, st, x, M, K, ldx,
                           scale, x8, ldx8);
    return launch_status();
}

}  // namespace

int launch_act_amax(const void* x, w4a8_dtype dt, int64_t M, int64_t K, int64_t ldx, float* amax, hipStream_t st) {
    int64_t blocks = (M * K + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    uint32_t* bits = reinterpret_cast<uint32_t*>(amax);
    if (dt == W4A8_F32)
        hipLaunchKernelGGL(act_amax_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const float*>(x), M, K,
                           ldx, bits);
    else
        hipLaunchKernelGGL(act_amax_kernel<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, st,
                           static_cast<const uint16_t*>(x), M, K, ldx, bits);
    return launch_status();
}

int launch_act_scale(const float* amax, float* scale, hipStream_t st) {
    hipLaunchKernelGGL(act_scale_kernel, dim3(1), dim3(64), 0, st, amax, scale);
    return launch_status();
}

int launch_quantize_act(const void* x, w4a8_dtype dt, int64_t M, int64_t K, int64_t ldx, const float* scale,
                        uint8_t* x8, int64_t ldx8, hipStream_t st) {
    if (dt == W4A8_F32) return launch_t(static_cast<const float*>(x), M, K, ldx, scale, x8, ldx8, st);
    return launch_t(static_cast<const uint16_t*>(x), M, K, ldx, scale, x8, ldx8, st);
}

}  // namespace w4a8
