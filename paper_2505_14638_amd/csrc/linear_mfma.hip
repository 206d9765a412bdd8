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
// a hand-laid software pipeline.
//   - Everything the main loop reads from global memory travels global -> LDS without passing through registers
//     (lds_dma_*): the activation block of the next chunk (shared, double buffered), and -- into slots private to
//     each wavefront -- the raw nibbles and the group scales of the band one chunk further ahead.  The loop therefore
//     holds no register-destination global load, and the only wait for memory is one `vmcnt(0)` at the end of a chunk,
//     a full chunk of MFMAs after the copies were issued.
//   - The nibble expansion of the NEXT chunk's band is spread over the sixteen MFMAs of the current chunk (one dword
//     every fourth MFMA) instead of running as a burst that idles the matrix unit.  Two operand buffers alternate by
//     chunk parity, so nothing is copied.
template <typename OutT>
__global__ void __launch_bounds__(512, 4) linear_mfma_tall_kernel(
    const uint8_t* __restrict__ x8, int M, int64_t ldx8, const float* __restrict__ s_x,
    const uint8_t* __restrict__ packed, const float* __restrict__ scales, int N, int n_tiles, int C, int cpg, int NG,
    OutT* __restrict__ y, int64_t ldy, int grid_m, int grid_n) {
    constexpr int WAVES = 8, MF = 16, BN = 128, BM = 256, STAGE_BYTES = BM * 128, DMA_PER_WAVE = 4;
    constexpr int RAW_OFF = 2 * STAGE_BYTES;                     // per wavefront: 1 KiB of raw nibbles (one tile)
    constexpr int SC_OFF = RAW_OFF + WAVES * 1024;               // per wavefront: 256 B, the band's 16 scales x 4 copies
    constexpr int LDS_BYTES = SC_OFF + WAVES * 256;
    constexpr int RS = BN + 16 / sizeof(OutT);
    constexpr int SLAB16_BYTES = 16 * RS * (int)sizeof(OutT);
    constexpr int FR = (RAW_OFF / SLAB16_BYTES < MF) ? RAW_OFF / SLAB16_BYTES : MF;
    __shared__ __attribute__((aligned(16))) uint8_t lds[LDS_BYTES];
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

    // wave-uniform bases (scalar registers) and small per-lane offsets
    const uint8_t* wbase = packed + (int64_t)t * C * 1024;       // + c * 1024 + lane * 16
    const uint8_t* sbase = reinterpret_cast<const uint8_t*>(scales) + (int64_t)t * NG * 64;   // + g * 64 + i * 4
    const uint8_t* xrow0 = x8 + (int64_t)m0 * ldx8;              // + c * 128 + xvoff
    const uint32_t woff = lane * 16, soff = i * 4;
    // Activation block in LDS: 16-token block f = 2 KiB = two 1 KiB pages of 8 rows x 128 bytes; 16-byte segment sg
    // (0..7) of row r (0..15) sits in page r / 8 at slot (r % 8) * 8 + (sg ^ ((r >> 1) & 7)).  One copy instruction
    // fills one page from eight whole 128-byte row segments of global memory (whole cache lines: the L2 -> CU path
    // moves about 2.5x more bytes per clock than with half lines), and the swizzle makes the two ds_read_b128 of an
    // operand (segments 2kq, 2kq+1 of row i, sixteen rows per quarter-wave) conflict-free.
    uint32_t xvoff[DMA_PER_WAVE];
#pragma unroll
    for (int q = 0; q < DMA_PER_WAVE; ++q) {
        const int d = wave * DMA_PER_WAVE + q;                   // page index: f = d / 2, rows 8 * (d % 2) .. + 7
        const int r = (d & 1) * 8 + (lane >> 3);
        const int sg = (lane & 7) ^ ((r >> 1) & 7);
        const int row = (d >> 1) * 16 + r;
        xvoff[q] = (uint32_t)(min(m0 + row, M - 1) - m0) * (uint32_t)ldx8 + sg * 16;
    }
    const uint32_t xa_off = (i >> 3) * 1024 + ((i & 7) * 8 + ((2 * kq) ^ ((i >> 1) & 7))) * 16;
    const uint32_t xc_off = (i >> 3) * 1024 + ((i & 7) * 8 + ((2 * kq + 1) ^ ((i >> 1) & 7))) * 16;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;
    const uint32_t lds_x = lds0 + (uint32_t)wave * (DMA_PER_WAVE * 1024);
    const uint32_t lds_raw = lds0 + RAW_OFF + (uint32_t)wave * 1024, lds_sc = lds0 + SC_OFF + (uint32_t)wave * 256;
    const uint8_t* my_raw = lds + RAW_OFF + wave * 1024 + lane * 16;
    const uint8_t* my_sc = lds + SC_OFF + wave * 256 + lane * 4;

    auto stage_x = [&](int c, int buf) {
        const uint8_t* xsrc = xrow0 + (int64_t)c * 128;
#pragma unroll
        for (int q = 0; q < DMA_PER_WAVE; ++q) lds_dma_16(xsrc, xvoff[q], lds_x + (uint32_t)buf * STAGE_BYTES + q * 1024);
    };
    // Copies the band's tile and scales of chunk c into the wavefront's slots.  `after` is a value read from those
    // slots earlier: the copy is issued only once that read has returned.
    auto stage_w = [&](int c, uint32_t after) {
        lds_dma_16_after(wbase + (int64_t)c * 1024, woff, lds_raw, after);
        lds_dma_4(sbase + (int64_t)(c / cpg) * 64, soff, lds_sc);
    };

    v4f acc[MF];
#pragma unroll
    for (int f = 0; f < MF; ++f) acc[f] = v4f{0.f, 0.f, 0.f, 0.f};

    // One chunk: multiply with `cur`; meanwhile read chunk c+1's nibbles and scale from the slots, expand them into
    // `next`, and start the copies of chunk c+2.
    auto chunk = [&](int c, const v8i& cur, float s_cur, v8i& next, float& s_next) {
        const int buf = c & 1;
        if (c + 1 < C) stage_x(c + 1, buf ^ 1);
        uint4 raw = make_uint4(0u, 0u, 0u, 0u);
        if (c + 1 < C) {
            raw = *reinterpret_cast<const uint4*>(my_raw);
            s_next = *reinterpret_cast<const float*>(my_sc);
            if (c + 2 < C) stage_w(c + 2, raw.x ^ __float_as_uint(s_next));
        }
        const uint32_t rn[4] = {raw.x, raw.y, raw.z, raw.w};
        const uint8_t* xb = lds + buf * STAGE_BYTES;
        uint4 xa = *reinterpret_cast<const uint4*>(xb + xa_off);
        uint4 xc = *reinterpret_cast<const uint4*>(xb + xc_off);
        // Step f: start the LDS reads of block f+1, issue the MFMA of block f, and fold the result of block f-1 (it
        // finished while this wavefront was waiting for its turn on the matrix unit) into the running sums.  The
        // scheduling fences keep the steps apart: without them the compiler batches all MFMAs before all FMAs and
        // needs sixteen result tiles of registers.
        v4f p_prev = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int f = 0; f < MF; ++f) {
            const v8i xop = v8i{(int)xa.x, (int)xa.y, (int)xa.z, (int)xa.w, (int)xc.x, (int)xc.y, (int)xc.z, (int)xc.w};
            if (f + 1 < MF) {
                xa = *reinterpret_cast<const uint4*>(xb + xa_off + (f + 1) * 2048);
                xc = *reinterpret_cast<const uint4*>(xb + xc_off + (f + 1) * 2048);
            }
            const v4f p = mfma_16x16x128_e4m3(xop, cur, v4f{0.f, 0.f, 0.f, 0.f});
            if (f > 0) {
                acc[f - 1][0] = fmaf(s_cur, p_prev[0], acc[f - 1][0]);
                acc[f - 1][1] = fmaf(s_cur, p_prev[1], acc[f - 1][1]);
                acc[f - 1][2] = fmaf(s_cur, p_prev[2], acc[f - 1][2]);
                acc[f - 1][3] = fmaf(s_cur, p_prev[3], acc[f - 1][3]);
                keep_here(acc[f - 1]);
            }
            if ((f & 1) == 1) {                                  // an eighth of the next band's expansion
                uint32_t e = (f & 2) ? nibbles_half_to_e4m3<4>(rn[f >> 2]) : nibbles_half_to_e4m3<0>(rn[f >> 2]);
                keep_here(e);
                next[f >> 1] = (int)e;
            }
            p_prev = p;
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // LDS reads of the next block
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // this block's MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, 12, 0);  // vector ALU work that does not depend on it
            __builtin_amdgcn_sched_barrier(0);
        }
        acc[MF - 1][0] = fmaf(s_cur, p_prev[0], acc[MF - 1][0]);
        acc[MF - 1][1] = fmaf(s_cur, p_prev[1], acc[MF - 1][1]);
        acc[MF - 1][2] = fmaf(s_cur, p_prev[2], acc[MF - 1][2]);
        acc[MF - 1][3] = fmaf(s_cur, p_prev[3], acc[MF - 1][3]);
        lds_dma_wait_all();                                      // this wavefront's copies have landed ...
        __syncthreads();                                         // ... and so have everyone's; the block just read is free
    };

    v8i wop_a, wop_b;
    float s_a, s_b = 0.f;
    {
        // chunk 0's band comes through registers, so that chunk 1's copies into the slots need not wait for it
        const uint4 raw0 = *reinterpret_cast<const uint4*>(wbase + woff);
        s_a = *reinterpret_cast<const float*>(sbase + soff);
        stage_x(0, 0);
        if (C > 1) stage_w(1, 0u);
        wop_a = slot_to_operand(raw0);
    }
    lds_dma_wait_all();
    __syncthreads();

    for (int c = 0; c < C; c += 2) {
        chunk(c, wop_a, s_a, wop_b, s_b);                        // even chunk: A multiplies, chunk c+1 expands into B
        if (c + 1 < C) chunk(c + 1, wop_b, s_b, wop_a, s_a);
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
    if (variant < 0 || variant > 6) return W4A8_ERR_SHAPE;      // 0 auto, 1 four-wave, 2 64x256, 3 128x256, 4 256x128
    const int C = (int)(K / 128), cpg = G / 128, NG = (int)(K / G);
    const int n_tiles = (int)((N + 15) / 16);
    // Workgroup shape.  Tall (256 tokens x 128 channels, one weight band per wavefront) amortizes the nibble expansion
    // over twice as many MFMAs and is the default; when that grid cannot fill the chip, shorter token blocks.
    int mf = 16, bn = 128;
    if (variant == 1 || variant == 3) { mf = 8; bn = 256; }
    bool pipelined = (variant == 5);
    if (variant == 2) { mf = 4; bn = 256; }
    if (variant == 6) { mf = 16; bn = 256; }
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
    } else if (variant == 6) {
        if (ydt == W4A8_F32) W4A8_LAUNCH_MFMA(float, 8, 2, 16, 256); else W4A8_LAUNCH_MFMA(uint16_t, 8, 2, 16, 256);
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
