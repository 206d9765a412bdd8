// W4A8 linear layer for many tokens (the compute-bound regime of Sec. 1): an MFMA-tiled GEMM with the INT4 -> E4M3
// expansion (Eq. 10) fused in front of the FP8 matrix unit.
//
// A workgroup computes a 128-token x 256-channel block of Y.  Each wavefront owns TPW 16-row weight tiles and all
// 128 tokens:
//   - weights never touch LDS: per 128-deep chunk a lane loads its 16-byte slot of each of its tiles straight
//     from the tiled format (coalesced 1 KiB reads), expands it once to 32 E4M3 bytes and reuses that operand for
//     all eight 16-token blocks;
//   - the activation block (128 tokens x 128 bytes) is shared by the wavefronts through LDS, double
//     buffered, filled by LDS-direct global loads (no staging registers) in MFMA operand order, so that the reads
//     are two conflict-free ds_read_b128 per operand;
//   - activations are the row operand and weights the column operand of the MFMA, so a result lane holds one
//     channel: its group scale is a single register, and every 16x16x128 MFMA (started from a zero accumulator)
//     is folded into the running sum with four FMAs against that scale -- group scales cannot be factored out
//     of the sum over K;
//   - the block of Y goes through LDS once at the end so that global stores are whole row segments.
// The FMAs and the nibble expansion keep the vector ALU about as busy as the matrix unit; the kernel relies on
// several resident wavefronts per SIMD (small register tiles) so that one wavefront's MFMAs overlap another's ALU work.
// Workgroups are numbered so that the ones resident on one XCD (one L2) at a time cover a compact rectangle of
// token blocks x channel blocks.
#include "w4a8_device.hpp"
#include "w4a8_internal.hpp"

namespace w4a8 {
namespace {

constexpr int XCDS = 8;
constexpr int GROUP_M = 8;          // token blocks per super-column of the block order

// WAVES wavefronts per workgroup, each owning TPW = 16 / WAVES weight tiles (WN = 16 * TPW channels); OCC = wavefronts
// per SIMD the register budget is sized for.
// MF 16-token operand blocks per workgroup (BM = 16 * MF tokens), BN channels per workgroup.
template <typename OutT, int WAVES, int OCC, int MF, int BN>
__global__ void __launch_bounds__(WAVES * 64, OCC) linear_mfma_kernel(
    const uint8_t* __restrict__ x8, int M, int64_t ldx8, const float* __restrict__ s_x,
    const uint8_t* __restrict__ packed, const float* __restrict__ scales, int N, int n_tiles, int C, int cpg, int NG,
    OutT* __restrict__ y, int64_t ldy, int grid_m, int grid_n) {
    constexpr int BM = 16 * MF, STAGE_BYTES = BM * 128;
    constexpr int TPW = (BN / 16) / WAVES, WN = TPW * 16;
    static_assert((2 * MF) % WAVES == 0, "activation half-blocks must divide evenly among the wavefronts");
    constexpr int DMA_PER_WAVE = (2 * MF) / WAVES;               // 1 KiB half-blocks of activations staged per wavefront
    constexpr int RS = BN + 16 / sizeof(OutT);                   // epilogue row stride: rows stay 16-byte aligned
    constexpr int SLAB16_BYTES = 16 * RS * (int)sizeof(OutT);    // one 16-token slab of the workgroup's output
    constexpr int LDS_BYTES = (2 * STAGE_BYTES > SLAB16_BYTES) ? 2 * STAGE_BYTES : SLAB16_BYTES;
    constexpr int FR = (LDS_BYTES / SLAB16_BYTES < MF) ? LDS_BYTES / SLAB16_BYTES : MF;   // slabs per epilogue round
    __shared__ __attribute__((aligned(16))) uint8_t lds[LDS_BYTES];
    uint8_t (*xs)[STAGE_BYTES] = reinterpret_cast<uint8_t (*)[STAGE_BYTES]>(lds);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kq = lane >> 4, i = lane & 15;

    // Block order.  Hardware deals consecutive workgroup ids round-robin to the eight XCDs; give each XCD a
    // contiguous range of the virtual order, and make the virtual order walk GROUP_M token blocks per channel block.
    const int total = grid_m * grid_n;
    const int per_xcd = (gridDim.x + XCDS - 1) / XCDS;
    const int v = (blockIdx.x % XCDS) * per_xcd + blockIdx.x / XCDS;
    if (v >= total) return;
    const int group = v / (GROUP_M * grid_n);
    const int first_m = group * GROUP_M;
    const int rows_in_group = min(GROUP_M, grid_m - first_m);
    const int in_group = v - group * GROUP_M * grid_n;
    const int bm = first_m + in_group % rows_in_group, bn = in_group / rows_in_group;
    const int m0 = bm * BM;
    const int t0 = bn * (BN / 16) + wave * TPW;

    const uint8_t* wbase[TPW];
    const uint8_t* sbase[TPW];
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        const int t = min(t0 + j, n_tiles - 1);                  // tiles past the end reload the last one; not stored
        wbase[j] = packed + (int64_t)t * C * 1024;
        sbase[j] = reinterpret_cast<const uint8_t*>(scales) + (int64_t)t * NG * 64;
    }
    const uint32_t woff = lane * 16, soff = i * 4;

    // activation staging: LDS-direct loads.  One wave-wide 16-byte load fills 1 KiB of LDS in lane order, which is
    // exactly one half (h) of one operand block (f): lane (kq, i) fetches bytes 32*kq + 16*h .. +15 of token row
    // 16*f + i.  The 16 half-blocks are dealt evenly to the wavefronts.  Rows past the end reload the last row; never stored.
    uint32_t xvoff[DMA_PER_WAVE];
#pragma unroll
    for (int q = 0; q < DMA_PER_WAVE; ++q) {
        const int d = wave * DMA_PER_WAVE + q;                   // half-block index: f = d / 2, h = d % 2
        const int row = (d >> 1) * 16 + i;
        xvoff[q] = (uint32_t)(min(m0 + row, M - 1) - m0) * (uint32_t)ldx8 + kq * 32 + (d & 1) * 16;
    }
    const uint8_t* xrow0 = x8 + (int64_t)m0 * ldx8;              // wave-uniform

    v4f acc[MF][TPW];
#pragma unroll
    for (int f = 0; f < MF; ++f)
#pragma unroll
        for (int j = 0; j < TPW; ++j) acc[f][j] = v4f{0.f, 0.f, 0.f, 0.f};

    uint4 wreg[TPW];
    float sreg[TPW];
    int g = 0, g_left = cpg;                                     // group of the chunk being loaded, chunks left in it
    auto global_loads = [&](int c, int buf) {
        const uint8_t* xsrc = xrow0 + (int64_t)c * 128;
#pragma unroll
        for (int q = 0; q < DMA_PER_WAVE; ++q)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(xsrc + xvoff[q]),
                (__attribute__((address_space(3))) void*)&xs[buf][(wave * DMA_PER_WAVE + q) * 1024], 16, 0, 0);
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            wreg[j] = *reinterpret_cast<const uint4*>(wbase[j] + (int64_t)c * 1024 + woff);
            sreg[j] = *reinterpret_cast<const float*>(sbase[j] + (int64_t)g * 64 + soff);
        }
        if (--g_left == 0) { ++g; g_left = cpg; }
    };

    global_loads(0, 0);
    __syncthreads();

    for (int c = 0; c < C; ++c) {
        const int buf = c & 1;
        v8i wop[TPW];
        float s[TPW];
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            wop[j] = slot_to_operand(wreg[j]);
            s[j] = sreg[j];
        }
        const bool more = (c + 1 < C);
        if (more) global_loads(c + 1, buf ^ 1);                  // lands while this chunk is being multiplied
        const uint8_t* xb = &xs[buf][lane * 16];
        uint4 xa = *reinterpret_cast<const uint4*>(xb);
        uint4 xc = *reinterpret_cast<const uint4*>(xb + 1024);
#pragma unroll
        for (int f = 0; f < MF; ++f) {
            const v8i xop = v8i{(int)xa.x, (int)xa.y, (int)xa.z, (int)xa.w, (int)xc.x, (int)xc.y, (int)xc.z, (int)xc.w};
            if (f + 1 < MF) {                                    // next block's operand is in flight during the MFMAs
                xa = *reinterpret_cast<const uint4*>(xb + (f + 1) * 2048);
                xc = *reinterpret_cast<const uint4*>(xb + (f + 1) * 2048 + 1024);
            }
#pragma unroll
            for (int j = 0; j < TPW; ++j) {
                // rows = tokens (activations), columns = channels (weights)
                const v4f p = mfma_16x16x128_e4m3(xop, wop[j], v4f{0.f, 0.f, 0.f, 0.f});
                acc[f][j][0] = fmaf(s[j], p[0], acc[f][j][0]);
                acc[f][j][1] = fmaf(s[j], p[1], acc[f][j][1]);
                acc[f][j][2] = fmaf(s[j], p[2], acc[f][j][2]);
                acc[f][j][3] = fmaf(s[j], p[3], acc[f][j][3]);
            }
        }
        __syncthreads();
    }

    // Epilogue.  Result lane: channel = lane % 16 of tile j, tokens 4*kq .. 4*kq+3 of block f.  The workgroup turns
    // FR 16-token slabs at a time into row-major order in LDS and stores whole BN-channel row segments.
    const float sx = *s_x;
    OutT* slab = reinterpret_cast<OutT*>(lds);
    constexpr int VEC = 16 / sizeof(OutT);                       // elements per 16-byte store
    constexpr int UPR = BN / VEC;                                // 16-byte units per row
    const int n_block = bn * BN;
    const bool vec_ok = (ldy % VEC == 0) && (reinterpret_cast<uintptr_t>(y) % 16 == 0);
#pragma unroll
    for (int f0 = 0; f0 < MF; f0 += FR) {
#pragma unroll
        for (int ff = 0; ff < FR; ++ff) {
            if (f0 + ff < MF) {
#pragma unroll
                for (int j = 0; j < TPW; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        slab[(ff * 16 + 4 * kq + r) * RS + wave * WN + 16 * j + i] =
                            OutCast<OutT>::cast(sx * acc[(f0 + ff < MF) ? f0 + ff : 0][j][r]);
            }
        }
        __syncthreads();
        constexpr int ROWS = FR * 16;
        for (int u = tid; u < ROWS * UPR; u += WAVES * 64) {
            const int row = u / UPR, col = (u % UPR) * VEC;
            const int m = m0 + f0 * 16 + row, n = n_block + col;
            if (row < (MF - f0) * 16 && m < M && n < N) {
                OutT* dst = y + (int64_t)m * ldy + n;
                const OutT* src = slab + row * RS + col;
                if (vec_ok && n + VEC <= N) {
                    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
                } else {
                    for (int e = 0; e < VEC && n + e < N; ++e) dst[e] = src[e];
                }
            }
        }
        __syncthreads();
    }
}

// The tall workgroup shape (256 tokens x 128 channels, eight wavefronts, one weight band each) as its own kernel with
// a hand-laid software pipeline: the nibble expansion of the NEXT chunk's band is spread over the sixteen MFMAs of the
// current chunk (one dword, 14 ALU ops, every fourth MFMA) instead of running as a burst that idles the matrix unit,
// and the raw nibbles are fetched two chunks ahead.  Two raw buffers and two operand buffers alternate by chunk
// parity, so nothing is copied.
template <typename OutT>
__global__ void __launch_bounds__(512, 4) linear_mfma_tall_kernel(
    const uint8_t* __restrict__ x8, int M, int64_t ldx8, const float* __restrict__ s_x,
    const uint8_t* __restrict__ packed, const float* __restrict__ scales, int N, int n_tiles, int C, int cpg, int NG,
    OutT* __restrict__ y, int64_t ldy, int grid_m, int grid_n) {
    constexpr int WAVES = 8, MF = 16, BN = 128, BM = 256, STAGE_BYTES = BM * 128, DMA_PER_WAVE = 4;
    constexpr int RS = BN + 16 / sizeof(OutT);
    constexpr int SLAB16_BYTES = 16 * RS * (int)sizeof(OutT);
    constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    constexpr int FR = (LDS_BYTES / SLAB16_BYTES < MF) ? LDS_BYTES / SLAB16_BYTES : MF;
    __shared__ __attribute__((aligned(16))) uint8_t lds[LDS_BYTES];
    uint8_t (*xs)[STAGE_BYTES] = reinterpret_cast<uint8_t (*)[STAGE_BYTES]>(lds);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kq = lane >> 4, i = lane & 15;

    const int total = grid_m * grid_n;
    const int per_xcd = (gridDim.x + XCDS - 1) / XCDS;
    const int v = (blockIdx.x % XCDS) * per_xcd + blockIdx.x / XCDS;
    if (v >= total) return;
    const int group = v / (GROUP_M * grid_n);
    const int first_m = group * GROUP_M;
    const int rows_in_group = min(GROUP_M, grid_m - first_m);
    const int in_group = v - group * GROUP_M * grid_n;
    const int bm = first_m + in_group % rows_in_group, bn = in_group / rows_in_group;
    const int m0 = bm * BM;
    const int t = min(bn * (BN / 16) + wave, n_tiles - 1);       // bands past the end reload the last one; not stored

    const uint8_t* wbase = packed + (int64_t)t * C * 1024 + lane * 16;
    const uint8_t* sbase = reinterpret_cast<const uint8_t*>(scales) + (int64_t)t * NG * 64 + i * 4;
    uint32_t xvoff[DMA_PER_WAVE];
#pragma unroll
    for (int q = 0; q < DMA_PER_WAVE; ++q) {
        const int d = wave * DMA_PER_WAVE + q;                   // half-block index: f = d / 2, h = d % 2
        const int row = (d >> 1) * 16 + i;
        xvoff[q] = (uint32_t)(min(m0 + row, M - 1) - m0) * (uint32_t)ldx8 + kq * 32 + (d & 1) * 16;
    }
    const uint8_t* xrow0 = x8 + (int64_t)m0 * ldx8;

    auto stage_x = [&](int c, int buf) {
        const uint8_t* xsrc = xrow0 + (int64_t)c * 128;
#pragma unroll
        for (int q = 0; q < DMA_PER_WAVE; ++q)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(xsrc + xvoff[q]),
                (__attribute__((address_space(3))) void*)&xs[buf][(wave * DMA_PER_WAVE + q) * 1024], 16, 0, 0);
    };
    int g = 0, g_left = cpg;                                     // group of the next chunk to be fetched
    int c_fetch = 0;
    auto fetch_w = [&](uint4& raw, float& s) {                   // raw nibbles and scale of chunk c_fetch, then advance
        raw = *reinterpret_cast<const uint4*>(wbase + (int64_t)c_fetch * 1024);
        s = *reinterpret_cast<const float*>(sbase + (int64_t)g * 64);
        ++c_fetch;
        if (--g_left == 0) { ++g; g_left = cpg; }
    };

    v4f acc[MF];
#pragma unroll
    for (int f = 0; f < MF; ++f) acc[f] = v4f{0.f, 0.f, 0.f, 0.f};

    // One chunk: multiply with `cur`; meanwhile expand `raw_next` (chunk c+1) into `next` and fetch chunk c+2 into `raw_far`.
    auto chunk = [&](int c, const v8i& cur, float s_cur, const uint4& raw_next, v8i& next, uint4& raw_far, float& s_far) {
        const int buf = c & 1;
        if (c + 1 < C) stage_x(c + 1, buf ^ 1);
        if (c + 2 < C) fetch_w(raw_far, s_far);
        const uint8_t* xb = &xs[buf][lane * 16];
        uint4 xa = *reinterpret_cast<const uint4*>(xb);
        uint4 xc = *reinterpret_cast<const uint4*>(xb + 1024);
        const uint32_t rn[4] = {raw_next.x, raw_next.y, raw_next.z, raw_next.w};
#pragma unroll
        for (int f = 0; f < MF; ++f) {
            const v8i xop = v8i{(int)xa.x, (int)xa.y, (int)xa.z, (int)xa.w, (int)xc.x, (int)xc.y, (int)xc.z, (int)xc.w};
            if (f + 1 < MF) {
                xa = *reinterpret_cast<const uint4*>(xb + (f + 1) * 2048);
                xc = *reinterpret_cast<const uint4*>(xb + (f + 1) * 2048 + 1024);
            }
            const v4f p = mfma_16x16x128_e4m3(xop, cur, v4f{0.f, 0.f, 0.f, 0.f});
            if ((f & 3) == 1) {                                  // a quarter of the next band's expansion
                uint32_t lo, hi;
                nibbles_to_e4m3(rn[f >> 2], lo, hi);
                next[2 * (f >> 2)] = (int)lo;
                next[2 * (f >> 2) + 1] = (int)hi;
            }
            acc[f][0] = fmaf(s_cur, p[0], acc[f][0]);
            acc[f][1] = fmaf(s_cur, p[1], acc[f][1]);
            acc[f][2] = fmaf(s_cur, p[2], acc[f][2]);
            acc[f][3] = fmaf(s_cur, p[3], acc[f][3]);
        }
        __syncthreads();
    };

    uint4 raw_a, raw_b = make_uint4(0u, 0u, 0u, 0u);
    float s_raw_a = 0.f, s_raw_b = 0.f;
    v8i wop_a, wop_b;
    stage_x(0, 0);
    fetch_w(raw_a, s_raw_a);                                     // chunk 0
    if (C > 1) fetch_w(raw_b, s_raw_b);                          // chunk 1
    wop_a = slot_to_operand(raw_a);
    float s_a = s_raw_a, s_b = 0.f;
    __syncthreads();

    for (int c = 0; c < C; c += 2) {
        // even chunk: operand A multiplies, raw B (chunk c+1) expands into operand B, chunk c+2 lands in raw A
        s_b = s_raw_b;
        chunk(c, wop_a, s_a, raw_b, wop_b, raw_a, s_raw_a);
        if (c + 1 < C) {
            s_a = s_raw_a;
            chunk(c + 1, wop_b, s_b, raw_a, wop_a, raw_b, s_raw_b);
        }
    }

    const float sx = *s_x;
    OutT* slab = reinterpret_cast<OutT*>(lds);
    constexpr int VEC = 16 / sizeof(OutT);
    constexpr int UPR = BN / VEC;
    const int n_block = bn * BN;
    const bool vec_ok = (ldy % VEC == 0) && (reinterpret_cast<uintptr_t>(y) % 16 == 0);
#pragma unroll
    for (int f0 = 0; f0 < MF; f0 += FR) {
#pragma unroll
        for (int ff = 0; ff < FR; ++ff) {
            if (f0 + ff < MF) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    slab[(ff * 16 + 4 * kq + r) * RS + wave * 16 + i] =
                        OutCast<OutT>::cast(sx * acc[(f0 + ff < MF) ? f0 + ff : 0][r]);
            }
        }
        __syncthreads();
        constexpr int ROWS = FR * 16;
        for (int u = tid; u < ROWS * UPR; u += WAVES * 64) {
            const int row = u / UPR, col = (u % UPR) * VEC;
            const int m = m0 + f0 * 16 + row, n = n_block + col;
            if (row < (MF - f0) * 16 && m < M && n < N) {
                OutT* dst = y + (int64_t)m * ldy + n;
                const OutT* src = slab + row * RS + col;
                if (vec_ok && n + VEC <= N) {
                    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
                } else {
                    for (int e = 0; e < VEC && n + e < N; ++e) dst[e] = src[e];
                }
            }
        }
        __syncthreads();
    }
}

}  // namespace

int launch_linear_mfma_tiled(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x,
                             const uint8_t* packed, const float* scales, int64_t N, int32_t G, void* y,
                             w4a8_dtype ydt, int64_t ldy, int variant, hipStream_t st) {
    if (variant < 0 || variant > 5) return W4A8_ERR_SHAPE;      // 0 auto, 1 four-wave, 2 64x256, 3 128x256, 4 256x128
    const int C = (int)(K / 128), cpg = G / 128, NG = (int)(K / G);
    const int n_tiles = (int)((N + 15) / 16);
    // Workgroup shape.  Tall (256 tokens x 128 channels, one weight band per wavefront) amortizes the nibble expansion
    // over twice as many MFMAs and is the default; when that grid cannot fill the chip, shorter token blocks.
    int mf = 16, bn = 128;
    if (variant == 1 || variant == 3) { mf = 8; bn = 256; }
    bool pipelined = (variant == 5);
    if (variant == 2) { mf = 4; bn = 256; }
    if (variant == 0) {
        const int64_t wg_tall = ((M + 255) / 256) * (int64_t)((n_tiles * 16 + 127) / 128);
        const int64_t wg_mid = ((M + 127) / 128) * (int64_t)((n_tiles * 16 + 255) / 256);
        if (wg_tall < 384) { mf = 8; bn = 256; if (wg_mid < 384) mf = 4; }
        else pipelined = true;
    }
    const int grid_n = (n_tiles * 16 + bn - 1) / bn;
    const int bm = 16 * mf;
    const int grid_m = (int)((M + bm - 1) / bm);
    const int64_t total = (int64_t)grid_m * grid_n;
    if (total > (1 << 30)) return W4A8_ERR_SHAPE;
    if (ldx8 >= (1 << 24)) return W4A8_ERR_SHAPE;               // 32-bit activation offsets inside a token block
    const dim3 grid((unsigned)((total + XCDS - 1) / XCDS * XCDS));
#define W4A8_LAUNCH_MFMA(T, WV, OC, MFV, BNV)                                                                        \
    hipLaunchKernelGGL((linear_mfma_kernel<T, WV, OC, MFV, BNV>), grid, dim3(WV * 64), 0, st, x8, (int)M, ldx8, s_x, \
                       packed, scales, (int)N, n_tiles, C, cpg, NG, static_cast<T*>(y), ldy, grid_m, grid_n)
    if (pipelined) {
        if (ydt == W4A8_F32)
            hipLaunchKernelGGL(linear_mfma_tall_kernel<float>, grid, dim3(512), 0, st, x8, (int)M, ldx8, s_x, packed, scales,
                               (int)N, n_tiles, C, cpg, NG, static_cast<float*>(y), ldy, grid_m, grid_n);
        else
            hipLaunchKernelGGL(linear_mfma_tall_kernel<uint16_t>, grid, dim3(512), 0, st, x8, (int)M, ldx8, s_x, packed,
                               scales, (int)N, n_tiles, C, cpg, NG, static_cast<uint16_t*>(y), ldy, grid_m, grid_n);
    } else if (variant == 1) {
        if (ydt == W4A8_F32) W4A8_LAUNCH_MFMA(float, 4, 2, 8, 256); else W4A8_LAUNCH_MFMA(uint16_t, 4, 2, 8, 256);
    } else if (mf == 16) {
        if (ydt == W4A8_F32) W4A8_LAUNCH_MFMA(float, 8, 4, 16, 128); else W4A8_LAUNCH_MFMA(uint16_t, 8, 4, 16, 128);
    } else if (mf == 8) {
        if (ydt == W4A8_F32) W4A8_LAUNCH_MFMA(float, 8, 4, 8, 256); else W4A8_LAUNCH_MFMA(uint16_t, 8, 4, 8, 256);
    } else {
        if (ydt == W4A8_F32) W4A8_LAUNCH_MFMA(float, 8, 4, 4, 256); else W4A8_LAUNCH_MFMA(uint16_t, 8, 4, 4, 256);
    }
#undef W4A8_LAUNCH_MFMA
    return launch_status();
}

}  // namespace w4a8
