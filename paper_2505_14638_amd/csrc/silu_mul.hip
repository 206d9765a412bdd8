// h = bf16( silu(gate) * up ): the elementwise step between the gate|up and down projections of a decoder block;
// optionally followed in the same kernel by the down projection's activation quantization (Eq. 13) of that bf16 value.
#include "w4a8_device.hpp"
#include "w4a8_internal.hpp"

namespace w4a8 {
namespace {

__device__ __forceinline__ float silu_mul(float g, float u) { return silu_mul_f32(g, u); }

// Q = false: h is bf16.  Q = true: h is E4M3 bytes, nearest_E4M3(bf16(silu(gate) * up) / *q_scale).
template <bool Q>
__global__ void __launch_bounds__(256) silu_mul_kernel(const uint16_t* __restrict__ gu, int64_t M, int64_t F,
                                                       int64_t ldgu, void* __restrict__ h_out, int64_t ldh, int vec,
                                                       const float* __restrict__ q_scale) {
    uint16_t* h = static_cast<uint16_t*>(h_out);
    uint8_t* h8 = static_cast<uint8_t*>(h_out);
    const float qs = Q ? *q_scale : 1.0f;
    if (vec) {                                   // 8 elements per thread, 16-byte accesses
        const int64_t F8 = F >> 3, total = M * F8;
        for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < total; u += (int64_t)gridDim.x * blockDim.x) {
            const int64_t m = u / F8, f = (u - m * F8) * 8;
            const uint4 a = *reinterpret_cast<const uint4*>(gu + m * ldgu + f);
            const uint4 b = *reinterpret_cast<const uint4*>(gu + m * ldgu + F + f);
            const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
            uint32_t o[4];
            float r[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float r0 = silu_mul(__uint_as_float(aw[j] << 16), __uint_as_float(bw[j] << 16));
                const float r1 = silu_mul(__uint_as_float(aw[j] & 0xFFFF0000u), __uint_as_float(bw[j] & 0xFFFF0000u));
                o[j] = (uint32_t)f32_to_bf16_bits(r0) | ((uint32_t)f32_to_bf16_bits(r1) << 16);
                r[2 * j] = __uint_as_float(o[j] << 16);          // the bf16 values, as the quantizer would read them
                r[2 * j + 1] = __uint_as_float(o[j] & 0xFFFF0000u);
            }
            if (Q) {
                uint32_t lo = cvt2(r[0] / qs, r[1] / qs, 0u, false), hi = cvt2(r[4] / qs, r[5] / qs, 0u, false);
                lo = cvt2(r[2] / qs, r[3] / qs, lo, true);
                hi = cvt2(r[6] / qs, r[7] / qs, hi, true);
                *reinterpret_cast<uint2*>(h8 + m * ldh + f) = make_uint2(lo, hi);
            } else {
                *reinterpret_cast<uint4*>(h + m * ldh + f) = make_uint4(o[0], o[1], o[2], o[3]);
            }
        }
    } else {
        const int64_t total = M * F;
        for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < total; u += (int64_t)gridDim.x * blockDim.x) {
            const int64_t m = u / F, f = u - m * F;
            const uint16_t b = f32_to_bf16_bits(silu_mul(bf16_bits_to_f32(gu[m * ldgu + f]), bf16_bits_to_f32(gu[m * ldgu + F + f])));
            if (Q)
                h8[m * ldh + f] = quantize_one(bf16_bits_to_f32(b), qs);
            else
                h[m * ldh + f] = b;
        }
    }
}

}  // namespace

int launch_silu_mul(const void* gu, int64_t M, int64_t F, int64_t ldgu, void* h, int64_t ldh, const float* q_scale,
                    hipStream_t st) {
    const int vec = (F % 8 == 0) && (ldgu % 8 == 0) && (ldh % 8 == 0) && (reinterpret_cast<uintptr_t>(gu) % 16 == 0) &&
                    (reinterpret_cast<uintptr_t>(h) % (q_scale ? 8 : 16) == 0);
    const int64_t units = vec ? M * (F / 8) : M * F;
    int64_t blocks = (units + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (q_scale)
        hipLaunchKernelGGL(silu_mul_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st,
                           static_cast<const uint16_t*>(gu), M, F, ldgu, h, ldh, vec, q_scale);
    else
        hipLaunchKernelGGL(silu_mul_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st,
                           static_cast<const uint16_t*>(gu), M, F, ldgu, h, ldh, vec, q_scale);
    return launch_status();
}

}  // namespace w4a8
