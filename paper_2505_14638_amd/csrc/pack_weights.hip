// Weight packing: symmetric round-to-nearest INT4 (Eq. 1, symmetric case) or re-layout of given codes,
// into the canonical or the tiled storage format; the asymmetric format (Eq. 1 with unsigned codes and zero-points,
// Eq. 8-9) into its tiled storage; and the INT4 -> E4M3 test hooks (Eq. 10).
// Offline with respect to inference: written for exactness and simplicity, not speed.
#include "w4a8_device.hpp"
#include "w4a8_internal.hpp"

namespace w4a8 {
namespace {

struct Geometry {
    int64_t N, K, NG;      // rows, columns, groups per row
    int64_t Np;            // rows of the destination (padded to 16 for the tiled layout)
    int32_t G;
    int tiled;
};

__device__ __forceinline__ int64_t scale_index(const Geometry& g, int64_t n, int64_t grp) {
    return g.tiled ? ((n >> 4) * g.NG + grp) * 16 + (n & 15) : n * g.NG + grp;
}

// destination byte -> row and the two columns whose codes it holds (low nibble, high nibble)
__device__ __forceinline__ void byte_to_coords(const Geometry& g, int64_t b, int64_t& n, int64_t& k_lo, int64_t& k_hi) {
    if (g.tiled) {
        const int64_t tile = b >> 10, C = g.K >> 7;
        const int64_t t = tile / C, c = tile - t * C;
        const int within = (int)(b & 1023), slot = within >> 4, byte = within & 15;
        const int kq = slot >> 4, i = slot & 15, d = byte >> 2, bb = byte & 3;
        n = t * 16 + i;
        k_lo = c * 128 + kq * 32 + d * 8 + bb;
        k_hi = k_lo + 4;
    } else {
        const int64_t half = g.K >> 1;
        n = b / half;
        k_lo = (b - n * half) * 2;
        k_hi = k_lo + 1;
    }
}

// one wavefront per (row, group): s = max|W| / 7 -- with pow2, the smallest power of two not below that quotient
// (Sec. 2.2: power-of-two scaling factors) -- or 1 for an all-zero group; padding rows get 0
__global__ void __launch_bounds__(256) rtn_scales_kernel(const float* __restrict__ w, Geometry g, int pow2,
                                                         float* __restrict__ scales) {
    const int64_t wid = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (wid >= g.Np * g.NG) return;
    const int64_t n = wid / g.NG, grp = wid - n * g.NG;
    float amax = 0.0f;
    if (n < g.N) {
        const float* p = w + n * g.K + grp * g.G;
        for (int j = lane; j < g.G; j += 64) amax = fmaxf(amax, fabsf(p[j]));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    if (lane == 0) {
        float s = 0.0f;
        if (n < g.N) s = (amax == 0.0f) ? 1.0f : __fdiv_rn(amax, 7.0f);
        if (pow2 && n < g.N && amax != 0.0f) {
            int e;
            const float m = frexpf(s, &e);                       // s = m * 2^e, m in [0.5, 1)
            s = ldexpf(1.0f, m == 0.5f ? e - 1 : e);
        }
        scales[scale_index(g, n, grp)] = s;
    }
}

// One wavefront per (row, group): copies the magnitude of the given scale; in the tiled layout the sign bit marks the
// groups whose codes contain -8 (the one code the fast nibble expansion gets wrong, see w4a8_device.hpp).
__global__ void __launch_bounds__(256) copy_scales_kernel(const float* __restrict__ src, const int8_t* __restrict__ q,
                                                          Geometry g, float* __restrict__ scales) {
    const int64_t wid = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (wid >= g.Np * g.NG) return;
    const int64_t n = wid / g.NG, grp = wid - n * g.NG;
    bool m8 = false;
    if (g.tiled && n < g.N) {
        const int8_t* p = q + n * g.K + grp * g.G;
        for (int j = lane; j < g.G; j += 64) m8 |= ((p[j] & 0xF) == 0x8);
    }
    const bool any = __builtin_amdgcn_ballot_w64(m8) != 0;
    if (lane == 0) {
        float s = (n < g.N) ? fabsf(src[n * g.NG + grp]) : 0.0f;
        if (any) s = __uint_as_float(__float_as_uint(s) | 0x80000000u);
        scales[scale_index(g, n, grp)] = s;
    }
}

__device__ __forceinline__ int rtn_code(float w, float s) {
    float r = rintf(w / s);                      // float32 division, round half to even
    r = fminf(fmaxf(r, -8.0f), 7.0f);
    return (int)r;
}

// nibble of a code in [-8, 7]: two's complement (canonical) or sign-magnitude with -8 as 1000 (tiled)
__device__ __forceinline__ uint32_t nibble_of(int code, int tiled) {
    if (!tiled) return ((uint32_t)code) & 0xFu;
    if (code >= 0) return (uint32_t)code;
    return code == -8 ? 8u : (8u | (uint32_t)(-code));
}

// one thread per destination byte
template <bool FROM_F32>
__global__ void __launch_bounds__(256) pack_kernel(const void* __restrict__ src, Geometry g,
                                                   const float* __restrict__ scales, uint8_t* __restrict__ packed) {
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= g.Np * (g.K >> 1)) return;
    int64_t n, k_lo, k_hi;
    byte_to_coords(g, b, n, k_lo, k_hi);
    uint32_t lo = 0, hi = 0;
    if (n < g.N) {
        if (FROM_F32) {
            const float* w = static_cast<const float*>(src) + n * g.K;
            // round-to-nearest with s = max|W| / 7 never yields -8, so no scale needs a mark
            lo = nibble_of(rtn_code(w[k_lo], scales[scale_index(g, n, k_lo / g.G)]), g.tiled);
            hi = nibble_of(rtn_code(w[k_hi], scales[scale_index(g, n, k_hi / g.G)]), g.tiled);
        } else {
            const int8_t* q = static_cast<const int8_t*>(src) + n * g.K;
            lo = nibble_of((int)(int8_t)(((int)q[k_lo] << 28) >> 28), g.tiled);   // only the low nibble of the input counts
            hi = nibble_of((int)(int8_t)(((int)q[k_hi] << 28) >> 28), g.tiled);
        }
    }
    packed[b] = (uint8_t)(lo | (hi << 4));
}

// Asymmetric format, parameters: one wavefront per (row, group) writes the row's scale and zero-point into the 80-byte
// record of its (16-row band, group).  FROM_F32: lo = min(min W, 0), hi = max(max W, 0), s = (hi - lo) / 15 (1 for an
// all-zero group), z = round(-lo / s), all float32; otherwise the given scale and zero-point (kept to 0..15).
template <bool FROM_F32>
__global__ void __launch_bounds__(256) asym_params_kernel(const float* __restrict__ w, const float* __restrict__ src_scales,
                                                          const uint8_t* __restrict__ src_zeros, Geometry g,
                                                          uint8_t* __restrict__ params) {
    const int64_t wid = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (wid >= g.Np * g.NG) return;
    const int64_t n = wid / g.NG, grp = wid - n * g.NG;
    float s = 0.0f;
    uint32_t z = 0u;
    if (n < g.N) {
        if (FROM_F32) {
            float lo = 0.0f, hi = 0.0f;
            const float* p = w + n * g.K + grp * g.G;
            for (int j = lane; j < g.G; j += 64) {
                lo = fminf(lo, p[j]);
                hi = fmaxf(hi, p[j]);
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                lo = fminf(lo, __shfl_xor(lo, off, 64));
                hi = fmaxf(hi, __shfl_xor(hi, off, 64));
            }
            const float span = __fsub_rn(hi, lo);
            s = (span == 0.0f) ? 1.0f : __fdiv_rn(span, 15.0f);
            z = (uint32_t)fminf(fmaxf(rintf(__fdiv_rn(-lo, s)), 0.0f), 15.0f);
        } else {
            s = src_scales[n * g.NG + grp];
            z = min((uint32_t)src_zeros[n * g.NG + grp], 15u);
        }
    }
    if (lane == 0) {
        uint8_t* rec = params + ((n >> 4) * g.NG + grp) * ASYM_RECORD_BYTES;
        reinterpret_cast<float*>(rec)[n & 15] = s;
        rec[64 + (n & 15)] = (uint8_t)z;
    }
}

// nibble of an unsigned code in the asymmetric storage: u = 7.5 +- (m + 0.5), sign-magnitude (see w4a8_device.hpp)
__device__ __forceinline__ uint32_t asym_nibble(uint32_t u) { return u >= 8u ? u - 8u : 15u - u; }

// u = clamp(round(W / s + z), 0, 15): float32 division, float32 addition, round half to even
__device__ __forceinline__ uint32_t asym_code(float w, float s, uint32_t z) {
    const float r = rintf(__fadd_rn(__fdiv_rn(w, s), (float)z));
    return (uint32_t)fminf(fmaxf(r, 0.0f), 15.0f);
}

// asymmetric format, codes: one thread per destination byte of the tiled storage
template <bool FROM_F32>
__global__ void __launch_bounds__(256) pack_asym_kernel(const void* __restrict__ src, Geometry g,
                                                        const uint8_t* __restrict__ params, uint8_t* __restrict__ packed) {
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= g.Np * (g.K >> 1)) return;
    int64_t n, k_lo, k_hi;
    byte_to_coords(g, b, n, k_lo, k_hi);
    uint32_t lo = 0, hi = 0;                                     // padding rows: code 0
    if (n < g.N) {
        if (FROM_F32) {
            const float* w = static_cast<const float*>(src) + n * g.K;
            const uint8_t* rec_lo = params + ((n >> 4) * g.NG + k_lo / g.G) * ASYM_RECORD_BYTES;
            const uint8_t* rec_hi = params + ((n >> 4) * g.NG + k_hi / g.G) * ASYM_RECORD_BYTES;
            lo = asym_code(w[k_lo], reinterpret_cast<const float*>(rec_lo)[n & 15], rec_lo[64 + (n & 15)]);
            hi = asym_code(w[k_hi], reinterpret_cast<const float*>(rec_hi)[n & 15], rec_hi[64 + (n & 15)]);
        } else {
            const uint8_t* q = static_cast<const uint8_t*>(src) + n * g.K;
            lo = q[k_lo] & 0xFu;                                 // only the low nibble of the input counts
            hi = q[k_hi] & 0xFu;
        }
    }
    packed[b] = (uint8_t)(asym_nibble(lo) | (asym_nibble(hi) << 4));
}

// tiled: one thread per 16-byte slot -> 32 consecutive bytes of one row of w8
// scales8 != nullptr: two-level bytes nearest_E4M3(code * s8[n, g]) with the tiled scale buffer of group size G
// asym_params != nullptr: asymmetric format, bytes nearest_E4M3(code - zero_point[n, g])
__global__ void __launch_bounds__(256) dequant_tiled_kernel(const uint4* __restrict__ packed, int64_t N, int64_t K,
                                                            int64_t slots, uint8_t* __restrict__ w8,
                                                            const float* __restrict__ scales8,
                                                            const uint8_t* __restrict__ asym_params, int asym_two_level,
                                                            int32_t G) {
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= slots) return;
    const int64_t tile = u >> 6, C = K >> 7;
    const int64_t t = tile / C, c = tile - t * C;
    const int slot = (int)(u & 63), kq = slot >> 4, i = slot & 15;
    const int64_t n = t * 16 + i;
    if (n >= N) return;
    v8i op;
    if (scales8) {
        const int64_t NG = K / G, grp = (c * 128) / G;
        op = slot_to_operand_two_level<true>(packed[u], two_level_table(scales8[(t * NG + grp) * 16 + i]));
    } else if (asym_params) {
        const int64_t NG = K / G, grp = (c * 128) / G;
        const uint8_t* rec = asym_params + (t * NG + grp) * ASYM_RECORD_BYTES;
        op = slot_to_operand_asym(packed[u], asym_two_level ? asym_two_level_table(rec[64 + i], reinterpret_cast<const float*>(rec)[i])
                                                            : asym_table(rec[64 + i]));
    } else {
        op = slot_to_operand<true>(packed[u]);
    }
    uint4* dst = reinterpret_cast<uint4*>(w8 + n * K + c * 128 + kq * 32);
    dst[0] = make_uint4((uint32_t)op[0], (uint32_t)op[1], (uint32_t)op[2], (uint32_t)op[3]);
    dst[1] = make_uint4((uint32_t)op[4], (uint32_t)op[5], (uint32_t)op[6], (uint32_t)op[7]);
}

// canonical: one thread per packed byte (two codes)
__global__ void __launch_bounds__(256) dequant_canonical_kernel(const uint8_t* __restrict__ packed, int64_t bytes,
                                                                uint8_t* __restrict__ w8) {
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= bytes) return;
    uint32_t lo, hi;
    nibbles_to_e4m3((uint32_t)packed[b], lo, hi);
    w8[2 * b] = (uint8_t)(lo & 0xFFu);
    w8[2 * b + 1] = (uint8_t)(hi & 0xFFu);
}

inline unsigned blocks_for(int64_t threads) { return (unsigned)((threads + 255) / 256); }

}  // namespace

int launch_pack_weights(const void* src, w4a8_src kind, const float* src_scales, int64_t N, int64_t K, int32_t G,
                        w4a8_layout layout, uint8_t* packed, float* scales, hipStream_t st) {
    Geometry g;
    g.N = N; g.K = K; g.G = G; g.NG = K / G;
    g.tiled = (layout == W4A8_LAYOUT_TILED);
    g.Np = g.tiled ? ((N + 15) / 16) * 16 : N;
    const int64_t n_scales = g.Np * g.NG, n_bytes = g.Np * (K / 2);
    if (kind == W4A8_SRC_F32_RTN || kind == W4A8_SRC_F32_RTN_POW2) {
        hipLaunchKernelGGL(rtn_scales_kernel, dim3(blocks_for(n_scales * 64)), dim3(256), 0, st,
                           static_cast<const float*>(src), g, kind == W4A8_SRC_F32_RTN_POW2 ? 1 : 0, scales);
        if (int e = launch_status()) return e;
        hipLaunchKernelGGL(pack_kernel<true>, dim3(blocks_for(n_bytes)), dim3(256), 0, st, src, g, scales, packed);
    } else {
        hipLaunchKernelGGL(copy_scales_kernel, dim3(blocks_for(n_scales * 64)), dim3(256), 0, st, src_scales,
                           static_cast<const int8_t*>(src), g, scales);
        if (int e = launch_status()) return e;
        hipLaunchKernelGGL(pack_kernel<false>, dim3(blocks_for(n_bytes)), dim3(256), 0, st, src, g, scales, packed);
    }
    return launch_status();
}

int launch_pack_weights_asym(const void* src, w4a8_src kind, const float* src_scales, const uint8_t* src_zeros,
                             int64_t N, int64_t K, int32_t G, uint8_t* packed, uint8_t* params, hipStream_t st) {
    Geometry g;
    g.N = N; g.K = K; g.G = G; g.NG = K / G;
    g.tiled = 1;
    g.Np = ((N + 15) / 16) * 16;
    const int64_t n_groups = g.Np * g.NG, n_bytes = g.Np * (K / 2);
    if (kind == W4A8_SRC_F32_RTN) {
        hipLaunchKernelGGL(asym_params_kernel<true>, dim3(blocks_for(n_groups * 64)), dim3(256), 0, st,
                           static_cast<const float*>(src), nullptr, nullptr, g, params);
        if (int e = launch_status()) return e;
        hipLaunchKernelGGL(pack_asym_kernel<true>, dim3(blocks_for(n_bytes)), dim3(256), 0, st, src, g, params, packed);
    } else {
        hipLaunchKernelGGL(asym_params_kernel<false>, dim3(blocks_for(n_groups * 64)), dim3(256), 0, st, nullptr,
                           src_scales, src_zeros, g, params);
        if (int e = launch_status()) return e;
        hipLaunchKernelGGL(pack_asym_kernel<false>, dim3(blocks_for(n_bytes)), dim3(256), 0, st, src, g, params, packed);
    }
    return launch_status();
}

int launch_dequant_weights(const uint8_t* packed, int64_t N, int64_t K, w4a8_layout layout, uint8_t* w8,
                           const float* scales8, const uint8_t* asym_params, int asym_two_level, int32_t G,
                           hipStream_t st) {
    if (layout == W4A8_LAYOUT_TILED) {
        const int64_t slots = ((N + 15) / 16) * (K / 128) * 64;
        hipLaunchKernelGGL(dequant_tiled_kernel, dim3(blocks_for(slots)), dim3(256), 0, st,
                           reinterpret_cast<const uint4*>(packed), N, K, slots, w8, scales8, asym_params, asym_two_level, G);
    } else {
        const int64_t bytes = N * (K / 2);
        hipLaunchKernelGGL(dequant_canonical_kernel, dim3(blocks_for(bytes)), dim3(256), 0, st, packed, bytes, w8);
    }
    return launch_status();
}

}  // namespace w4a8
