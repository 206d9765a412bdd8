// W4A8 linear layer for many tokens (the compute-bound regime of Sec. 1): an MFMA-tiled GEMM with the INT4 -> E4M3
// expansion (Eq. 10) fused in front of the FP8 matrix unit.
//
// A workgroup of four wavefronts computes a 128-token x 256-channel block of Y.  Each wavefront owns 64 channels
// (four 16-row weight tiles) and all 128 tokens:
//   - weights never touch LDS: per 128-deep chunk a lane loads its 16-byte slot of each of the four tiles straight
//     from the tiled format (coalesced 1 KiB reads), expands it once to 32 E4M3 bytes and reuses that A operand for
//     all eight 16-token blocks;
//   - the activation block (128 tokens x 128 bytes) is shared by the four wavefronts through LDS, double
//     buffered, stored in MFMA operand order so that the reads are two conflict-free ds_read_b128 per operand;
//   - every 16x16x128 MFMA starts from a zero accumulator and its result is folded into the running sum with the
//     fp32 group scale of the channel (four FMAs per MFMA), because group scales cannot be factored out of K.
#include "w4a8_device.hpp"
#include "w4a8_internal.hpp"

namespace w4a8 {
namespace {

constexpr int BM = 128;             // tokens per workgroup
constexpr int WAVES = 4;
constexpr int TPW = 4;              // weight tiles (16 channels each) per wavefront
constexpr int BN = WAVES * TPW * 16;
constexpr int MF = BM / 16;         // 16-token operand blocks per workgroup
constexpr int STAGE_BYTES = BM * 128;

// LDS position of the 16-byte unit (row, u) of an activation block: operand order.
// u = 2*kq + h: the lane (kq, row % 16) of block row / 16 reads halves h = 0, 1 at +0 and +1024.
__device__ __forceinline__ int lds_unit_offset(int row, int u) {
    return (row >> 4) * 2048 + (u & 1) * 1024 + ((u >> 1) * 16 + (row & 15)) * 16;
}

template <typename OutT>
__global__ void __launch_bounds__(WAVES * 64) linear_mfma_kernel(
    const uint8_t* __restrict__ x8, int M, int64_t ldx8, const float* __restrict__ s_x,
    const uint4* __restrict__ packed, const float* __restrict__ scales, int N, int n_tiles, int C, int cpg, int NG,
    OutT* __restrict__ y, int64_t ldy, int grid_m, int grid_n) {
    __shared__ __attribute__((aligned(16))) uint8_t xs[2][STAGE_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kq = lane >> 4, i = lane & 15;

    // block order: token blocks fastest, so that workgroups in flight together share weight tiles in L2
    const int bm = blockIdx.x % grid_m, bn = blockIdx.x / grid_m;
    const int m0 = bm * BM;
    const int t0 = bn * (WAVES * TPW) + wave * TPW;

    const uint4* wp[TPW];
    const float4* sp[TPW];
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        const int t = min(t0 + j, n_tiles - 1);
        wp[j] = packed + (int64_t)t * C * 64 + lane;
        sp[j] = reinterpret_cast<const float4*>(scales + (int64_t)t * NG * 16 + 4 * kq);
    }

    // activation staging: thread -> (row within a pass of 32 rows, 16-byte unit); four passes cover 128 rows
    const int ld_row = tid >> 3, ld_u = tid & 7;
    const uint8_t* xg[4];
    int xo[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int row = p * 32 + ld_row;
        xg[p] = x8 + (int64_t)min(m0 + row, M - 1) * ldx8 + ld_u * 16;
        xo[p] = lds_unit_offset(row, ld_u);
    }

    v4f acc[MF][TPW];
#pragma unroll
    for (int f = 0; f < MF; ++f)
#pragma unroll
        for (int j = 0; j < TPW; ++j) acc[f][j] = v4f{0.f, 0.f, 0.f, 0.f};

    uint4 xreg[4], wreg[TPW];
    float4 sreg[TPW];
    auto global_loads = [&](int c) {
#pragma unroll
        for (int p = 0; p < 4; ++p) xreg[p] = *reinterpret_cast<const uint4*>(xg[p] + (int64_t)c * 128);
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            wreg[j] = wp[j][(int64_t)c * 64];
            sreg[j] = sp[j][(c / cpg) * 4];
        }
    };

    global_loads(0);
#pragma unroll
    for (int p = 0; p < 4; ++p) *reinterpret_cast<uint4*>(&xs[0][xo[p]]) = xreg[p];
    __syncthreads();

    for (int c = 0; c < C; ++c) {
        const int buf = c & 1;
        v8i wop[TPW];
        float4 s[TPW];
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            wop[j] = slot_to_operand(wreg[j]);
            s[j] = sreg[j];
        }
        const bool more = (c + 1 < C);
        if (more) global_loads(c + 1);
        const uint8_t* xb = &xs[buf][lane * 16];
#pragma unroll
        for (int f = 0; f < MF; ++f) {
            const uint4 a = *reinterpret_cast<const uint4*>(xb + f * 2048);
            const uint4 b = *reinterpret_cast<const uint4*>(xb + f * 2048 + 1024);
            const v8i xop = v8i{(int)a.x, (int)a.y, (int)a.z, (int)a.w, (int)b.x, (int)b.y, (int)b.z, (int)b.w};
#pragma unroll
            for (int j = 0; j < TPW; ++j) {
                const v4f p = mfma_16x16x128_e4m3(wop[j], xop, v4f{0.f, 0.f, 0.f, 0.f});
                acc[f][j][0] = fmaf(s[j].x, p[0], acc[f][j][0]);
                acc[f][j][1] = fmaf(s[j].y, p[1], acc[f][j][1]);
                acc[f][j][2] = fmaf(s[j].z, p[2], acc[f][j][2]);
                acc[f][j][3] = fmaf(s[j].w, p[3], acc[f][j][3]);
            }
        }
        if (more) {
#pragma unroll
            for (int p = 0; p < 4; ++p) *reinterpret_cast<uint4*>(&xs[buf ^ 1][xo[p]]) = xreg[p];
        }
        __syncthreads();
    }

    // result lane: token = lane % 16 of block f, channels 4*kq .. 4*kq+3 of tile j
    const float sx = *s_x;
#pragma unroll
    for (int f = 0; f < MF; ++f) {
        const int m = m0 + f * 16 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            const int n = (t0 + j) * 16 + 4 * kq;
            OutT* dst = y + (int64_t)m * ldy + n;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (n + r < N) dst[r] = OutCast<OutT>::cast(sx * acc[f][j][r]);
        }
    }
}

}  // namespace

int launch_linear_mfma_tiled(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x,
                             const uint8_t* packed, const float* scales, int64_t N, int32_t G, void* y,
                             w4a8_dtype ydt, int64_t ldy, int variant, hipStream_t st) {
    if (variant != 0) return W4A8_ERR_SHAPE;
    const int C = (int)(K / 128), cpg = G / 128, NG = (int)(K / G);
    const int n_tiles = (int)((N + 15) / 16);
    const int grid_m = (int)((M + BM - 1) / BM), grid_n = (n_tiles * 16 + BN - 1) / BN;
    const dim3 grid((unsigned)grid_m * (unsigned)grid_n), block(WAVES * 64);
    if (ydt == W4A8_F32)
        hipLaunchKernelGGL(linear_mfma_kernel<float>, grid, block, 0, st, x8, (int)M, ldx8, s_x,
                           reinterpret_cast<const uint4*>(packed), scales, (int)N, n_tiles, C, cpg, NG,
                           static_cast<float*>(y), ldy, grid_m, grid_n);
    else
        hipLaunchKernelGGL(linear_mfma_kernel<uint16_t>, grid, block, 0, st, x8, (int)M, ldx8, s_x,
                           reinterpret_cast<const uint4*>(packed), scales, (int)N, n_tiles, C, cpg, NG,
                           static_cast<uint16_t*>(y), ldy, grid_m, grid_n);
    return launch_status();
}

}  // namespace w4a8
