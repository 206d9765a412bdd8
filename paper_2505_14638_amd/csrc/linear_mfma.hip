// W4A8 linear layer for many tokens (the compute-bound regime of Sec. 1): an MFMA-tiled GEMM with the INT4 -> E4M3
// expansion (Eq. 10) fused in front of the FP8 matrix unit.
//
// A workgroup of eight wavefronts computes 16*MF tokens x (128 * TPW / KS) channels of Y.  The wavefronts form KS
// groups that split K between them: in every pass over the main loop group kg multiplies the 128-deep chunk
// c = KS * pass + kg.  Inside a group each wavefront owns TPW 16-channel weight bands and all 16*MF tokens:
//   - activations are the row operand and weights the column operand of the 16x16x128 MFMA, so a result lane holds
//     one channel: its group scale is a single register, and every MFMA (started from a zero accumulator) is folded
//     into the running sum with four FMAs against that scale -- group scales cannot be factored out of the sum over K;
//   - everything the main loop reads from global memory travels global -> LDS without passing through registers
//     (lds_dma_*): the activation block of the next pass (shared by the workgroup, double buffered) and -- into slots
//     private to each wavefront -- the raw nibbles and the group scales of the band one pass further ahead.  The loop
//     holds no register-destination global load, and its only wait for memory is one `vmcnt(0)` at the end of a
//     pass, a whole pass of MFMAs after the copies were issued;
//   - the band's nibbles are expanded once per chunk and reused for all MF token blocks; the expansion of the NEXT
//     chunk is spread over the MFMAs of the current one, and two operand buffers alternate by pass parity, so nothing
//     is copied;
//   - each step issues the LDS reads of the next token block, then this block's MFMA, then the FMAs of the previous
//     block (independent of the MFMA in flight); the steps of a pass form one basic block and run at raised wavefront
//     priority;
//   - the K-split groups add their partial sums through LDS, and the block of Y goes through LDS once more so that
//     global stores are whole row segments.
// Workgroups are numbered so that the ones resident on one XCD (one L2) at a time cover a compact rectangle of
// token blocks x channel blocks.
#include "w4a8_device.hpp"
#include "w4a8_internal.hpp"

namespace w4a8 {
namespace {

constexpr int XCDS = 8;
constexpr int GROUP_M = 8;          // token blocks per super-column of the block order
constexpr int WAVES = 8;

// Built workgroup shapes {token blocks, K-split groups, bands per wavefront}, in the launcher's order of preference
// (the last one is considered first, under its own condition).
#define W4A8_MFMA_SHAPES 7
#define W4A8_MFMA_SHAPE_LIST {{16, 1, 1}, {8, 1, 1}, {8, 2, 1}, {4, 1, 1}, {4, 2, 1}, {4, 4, 1}, {16, 1, 2}}

template <int A, int B> struct MaxOf { static constexpr int value = A > B ? A : B; };

// MODE_CODE_EXACT: signed codes, group scales applied to the partial sums in fp32.  MODE_TWO_LEVEL: the weight operand
// is nearest_E4M3(code * s8[n,g]) and the sum over all of K stays in the MFMA accumulator; the output is scaled by
// s_x * w_out[n] (w_out[0] when per_channel is 0).  MODE_ASYM: unsigned codes with per-group zero-points, the weight
// operand is the integer code - zero_point, group scales as in the code-exact mode; `scales` then points at the
// 80-byte records of scales and zero-points.  MODE_POW2: signed codes, the group scale is a power of two that the
// matrix unit applies itself (block-scaled MFMA), so the sum over all of K stays in the MFMA accumulator.
// MODE_ASYM_TWO: the asymmetric records with FP8-domain scales; the weight operand is
// nearest_E4M3((code - zero_point) * s8[n,g]), accumulation and output scale as in MODE_TWO_LEVEL.
template <typename OutT, int MF, int KS, int TPW, int MODE>
__global__ void __launch_bounds__(512, (KS * MF > 16 || MF * TPW > 16) ? 2 : 4) linear_mfma_kernel(
    const uint8_t* __restrict__ x8, int M, int64_t ldx8, const float* __restrict__ s_x,
    const uint8_t* __restrict__ packed, const float* __restrict__ scales, int N, int n_tiles, int C, int cpg, int NG,
    OutT* __restrict__ y, int64_t ldy, int grid_m, int grid_n, const float* __restrict__ w_out, int per_channel,
    const float* __restrict__ y_scale) {
    constexpr bool ASYM2 = MODE == MODE_ASYM_TWO;                // asymmetric records, two-level bytes
    constexpr bool TWO = MODE == MODE_TWO_LEVEL, ASYM = MODE == MODE_ASYM || ASYM2, POW2 = MODE == MODE_POW2;
    constexpr bool IN_MFMA = TWO || POW2 || ASYM2;               // the sum over K stays in the MFMA accumulator
    constexpr bool OUT_SCALED = TWO || ASYM2;                    // output scaled by s_x * w_out[n]
    constexpr int REC = ASYM ? ASYM_RECORD_BYTES : 64;           // bytes of scales (and zero-points) per band and group
    constexpr int NB = WAVES / KS;                               // wavefronts per K-split group, TPW weight bands each
    constexpr int BN = 16 * NB * TPW, BM = 16 * MF;
    constexpr int PAGES = KS * MF * 2;                           // 1 KiB pages of activations per pass
    constexpr int STAGE_BYTES = PAGES * 1024, DMA_PER_WAVE = PAGES / WAVES;
    static_assert(PAGES % WAVES == 0, "activation pages must divide evenly among the wavefronts");
    constexpr int RAW_OFF = 2 * STAGE_BYTES;                     // per wavefront and band: 1 KiB of raw nibbles (one tile)
    constexpr int SC_OFF = RAW_OFF + WAVES * TPW * 1024;         // per wavefront and band: 256 B, 16 scales x 4 copies
    constexpr int ZP_OFF = SC_OFF + WAVES * TPW * 256;           // asymmetric format: per lane the dword that holds its zero-point
    constexpr int LOOP_BYTES = ZP_OFF + (ASYM ? WAVES * TPW * 256 : 0);
    constexpr int RED_BYTES = (KS - 1) * NB * TPW * MF * 4 * 64 * 4;   // partial sums of groups 1 .. KS-1
    using SlabT = typename OutKind<OutT>::Slab;                  // element of the epilogue's LDS slab
    constexpr bool SILU = OutKind<OutT>::SILU;
    constexpr int RS = BN + 16 / sizeof(SlabT);                  // epilogue row stride: rows stay 16-byte aligned
    constexpr int SLAB16_BYTES = 16 * RS * (int)sizeof(SlabT);   // one 16-token slab of the workgroup's output
    constexpr int LDS_BYTES = MaxOf<MaxOf<LOOP_BYTES, RED_BYTES>::value, SLAB16_BYTES>::value;
    constexpr int FR = (LDS_BYTES / SLAB16_BYTES < MF) ? LDS_BYTES / SLAB16_BYTES : MF;   // slabs per epilogue round
    constexpr int PIECES = (8 + MF - 1) / MF;                    // eighths of a band's expansion per step, at most
    __shared__ __attribute__((aligned(16))) uint8_t lds[LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = wave / NB, band = wave % NB;
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

    // wave-uniform bases (scalar registers) and small per-lane offsets
    const uint8_t* wbase[TPW];                                   // + c * 1024 + lane * 16
    const uint8_t* sbase[TPW];                                   // + g * 64 + i * 4
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        const int t = min((bn * NB + band) * TPW + j, n_tiles - 1);   // bands past the end reload the last one; not stored
        wbase[j] = packed + (int64_t)t * C * 1024;
        sbase[j] = reinterpret_cast<const uint8_t*>(scales) + (int64_t)t * NG * REC;
    }
    const uint8_t* xrow0 = x8 + (int64_t)m0 * ldx8;              // + c * 128 + xvoff
    const uint32_t woff = lane * 16, soff = i * 4, zoff = 64 + (i >> 2) * 4;   // zoff: the dword with channel i's zero-point
    // Activation block in LDS: K-split group kg, 16-token block f = 2 KiB = two 1 KiB pages of 8 rows x 128 bytes;
    // 16-byte segment sg (0..7) of row r (0..15) sits in page r / 8 at slot (r % 8) * 8 + (sg ^ sw(r)) with
    // sw(r) = (r % 8) ^ (r / 8).  One copy instruction fills one page from eight whole 128-byte row segments of global
    // memory (whole cache lines).  The swizzle keeps the two ds_read_b128 of an operand (segments 2kq, 2kq+1 of row i)
    // free of bank conflicts whether the LDS serves eight consecutive lanes per clock from 32 banks or sixteen from 64:
    // any eight consecutive rows differ in slot % 8, any sixteen in slot % 16.  Page d of a pass belongs to group
    // d / (2 MF), block (d / 2) % MF, rows 8 (d % 2)..+7.
    uint32_t xvoff[DMA_PER_WAVE];
#pragma unroll
    for (int q = 0; q < DMA_PER_WAVE; ++q) {
        const int d = wave * DMA_PER_WAVE + q;
        const int r = (d & 1) * 8 + (lane >> 3);
        const int sg = (lane & 7) ^ ((r & 7) ^ (r >> 3));
        const int row = ((d >> 1) % MF) * 16 + r;
        xvoff[q] = (uint32_t)(min(m0 + row, M - 1) - m0) * (uint32_t)ldx8 + sg * 16;   // rows past the end: last row
    }
    const uint32_t xa_off = kg * (MF * 2048) + (i >> 3) * 1024 + ((i & 7) * 8 + ((2 * kq) ^ ((i & 7) ^ (i >> 3)))) * 16;
    const uint32_t xc_off = kg * (MF * 2048) + (i >> 3) * 1024 + ((i & 7) * 8 + ((2 * kq + 1) ^ ((i & 7) ^ (i >> 3)))) * 16;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;
    const uint32_t lds_x = lds0 + (uint32_t)wave * (DMA_PER_WAVE * 1024);
    const uint32_t lds_raw = lds0 + RAW_OFF + (uint32_t)wave * (TPW * 1024), lds_sc = lds0 + SC_OFF + (uint32_t)wave * (TPW * 256);
    const uint8_t* my_raw = lds + RAW_OFF + wave * (TPW * 1024) + lane * 16;      // + j * 1024
    const uint8_t* my_sc = lds + SC_OFF + wave * (TPW * 256) + lane * 4;          // + j * 256
    const uint32_t lds_zp = lds0 + ZP_OFF + (uint32_t)wave * (TPW * 256);
    const uint8_t* my_zp = lds + ZP_OFF + wave * (TPW * 256) + lane * 4;          // + j * 256

    const int passes = (C + KS - 1) / KS;
    // activations of pass `ps` into stage `buf`; chunks past the end of K reload the last chunk (never multiplied)
    auto stage_x = [&](int ps, int buf) {
#pragma unroll
        for (int q = 0; q < DMA_PER_WAVE; ++q) {
            const int d = wave * DMA_PER_WAVE + q;
            const int c = min(ps * KS + d / (2 * MF), C - 1);
            lds_dma_16(xrow0 + (int64_t)c * 128, xvoff[q], lds_x + (uint32_t)buf * STAGE_BYTES + q * 1024);
        }
    };
    // Copies the band's tile and scales of chunk c into the wavefront's slots.  `after` is a value read from those
    // slots earlier: the copy is issued only once that read has returned.
    auto stage_w = [&](int c, uint32_t after) {
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            lds_dma_16_after(wbase[j] + (int64_t)c * 1024, woff, lds_raw + j * 1024, after);
            lds_dma_4(sbase[j] + (int64_t)(c / cpg) * REC, soff, lds_sc + j * 256);
            if (ASYM) lds_dma_4(sbase[j] + (int64_t)(c / cpg) * REC, zoff, lds_zp + j * 256);
        }
    };

    v4f acc[MF][TPW];
#pragma unroll
    for (int f = 0; f < MF; ++f)
#pragma unroll
        for (int j = 0; j < TPW; ++j) acc[f][j] = v4f{0.f, 0.f, 0.f, 0.f};

    struct Band { v8i op[TPW]; float s[TPW]; };
    // One pass: multiply chunk c = KS * ps + kg with `cur`; meanwhile read chunk c + KS's nibbles and scales from the
    // slots, expand them into `next`, and start the copies of chunk c + 2 KS.
    auto pass = [&](int ps, const Band& cur, Band& next) {
        const int buf = ps & 1;
        const int c = ps * KS + kg;
        if (ps + 1 < passes) stage_x(ps + 1, buf ^ 1);
        uint4 raw[TPW];
#pragma unroll
        for (int j = 0; j < TPW; ++j) raw[j] = make_uint4(0u, 0u, 0u, 0u);
        bool m8[TPW];                                            // the band's next chunk lies in a group that holds -8
        uint32_t zp[TPW];                                        // asymmetric format: the lane's zero-point in the next chunk
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            m8[j] = false;
            zp[j] = 0u;
        }
        if (c + KS < C) {
            uint32_t seen = 0u;
#pragma unroll
            for (int j = 0; j < TPW; ++j) {
                raw[j] = *reinterpret_cast<const uint4*>(my_raw + j * 1024);
                next.s[j] = *reinterpret_cast<const float*>(my_sc + j * 256);
                seen ^= raw[j].x ^ __float_as_uint(next.s[j]);
                if (ASYM) {
                    const uint32_t zw = *reinterpret_cast<const uint32_t*>(my_zp + j * 256);
                    seen ^= zw;
                    zp[j] = (zw >> (8 * (i & 3))) & 0xFFu;
                } else {
                    m8[j] = any_marked(next.s[j]);
                }
            }
            if (c + 2 * KS < C) stage_w(c + 2 * KS, seen);
        }
        MagTable tab[TPW];                                       // two-level mode: the next chunk's magnitude tables
#pragma unroll
        for (int j = 0; j < TPW; ++j) tab[j] = TWO ? two_level_table(next.s[j]) : MagTable{0u, 0u, 0u};
        AsymTable atab[TPW];                                     // asymmetric format: the next chunk's code - zero_point bytes
#pragma unroll
        for (int j = 0; j < TPW; ++j)
            atab[j] = ASYM2 ? asym_two_level_table(zp[j], next.s[j]) : ASYM ? asym_table(zp[j]) : AsymTable{{0u, 0u, 0u, 0u}};
        if (c < C) {
            // The MFMA steps run at raised wavefront priority, the head of a pass (copies) and its end (wait, barrier)
            // at the default one: a wavefront that has MFMAs to issue then wins arbitration over one that is waiting
            // anyway.  Measured +2...8 % on the prefill shapes; raising it around the MFMA alone loses 1-3 %.
            __builtin_amdgcn_s_setprio(1);
            const uint8_t* xb = lds + buf * STAGE_BYTES;
            uint4 xa = *reinterpret_cast<const uint4*>(xb + xa_off);
            uint4 xc = *reinterpret_cast<const uint4*>(xb + xc_off);
            v4f p_prev = v4f{0.f, 0.f, 0.f, 0.f};
            // Step (f, j): the LDS reads of token block f+1 (at j = 0), the MFMA of block f with band j, then the FMAs
            // of the previous step, which do not depend on the MFMA in flight, and a share of the next chunk's expansion.
#pragma unroll
            for (int f = 0; f < MF; ++f) {
                const v8i xop = v8i{(int)xa.x, (int)xa.y, (int)xa.z, (int)xa.w, (int)xc.x, (int)xc.y, (int)xc.z, (int)xc.w};
                if (f + 1 < MF) {
                    xa = *reinterpret_cast<const uint4*>(xb + xa_off + (f + 1) * 2048);
                    xc = *reinterpret_cast<const uint4*>(xb + xc_off + (f + 1) * 2048);
                }
#pragma unroll
                for (int j = 0; j < TPW; ++j) {
                    const int st = f * TPW + j;                  // step number
                    if (TWO || ASYM2) acc[f][j] = mfma_16x16x128_e4m3(xop, cur.op[j], acc[f][j]);
                    if (POW2) acc[f][j] = mfma_16x16x128_e4m3_scaled(xop, cur.op[j], acc[f][j], E8M0_ONE, e8m0_of(cur.s[j]));
                    const v4f p = IN_MFMA ? v4f{0.f, 0.f, 0.f, 0.f} : mfma_16x16x128_e4m3(xop, cur.op[j], v4f{0.f, 0.f, 0.f, 0.f});
                    if (!IN_MFMA && st > 0) {
                        const int fp = (st - 1) / TPW, jp = (st - 1) % TPW;
                        const float sc = fabsf(cur.s[jp]);       // the sign bit is the packer's mark, not part of the scale
                        acc[fp][jp][0] = fmaf(sc, p_prev[0], acc[fp][jp][0]);
                        acc[fp][jp][1] = fmaf(sc, p_prev[1], acc[fp][jp][1]);
                        acc[fp][jp][2] = fmaf(sc, p_prev[2], acc[fp][jp][2]);
                        acc[fp][jp][3] = fmaf(sc, p_prev[3], acc[fp][jp][3]);
                        keep_here(acc[fp][jp]);
                    }
                    // this step's share of the next chunk's expansion: eighths st*8/MF .. (st+1)*8/MF - 1 of the 8 TPW;
                    // eighth E belongs to band E / 8 and is operand register e = E % 8: half e % 2 of dword e / 2
#pragma unroll
                    for (int E = st * 8 / MF; E < (st + 1) * 8 / MF; ++E) {
                        const int jb = E / 8, e = E % 8;
                        const int d = e >> 1;
                        const uint32_t src = d == 0 ? raw[jb].x : d == 1 ? raw[jb].y : d == 2 ? raw[jb].z : raw[jb].w;
                        uint32_t o;
                        if (TWO) {
                            o = (e & 1) ? two_level_half_fast<4>(src, tab[jb]) : two_level_half_fast<0>(src, tab[jb]);
                        } else if (ASYM) {
                            o = (e & 1) ? asym_half<4>(src, atab[jb]) : asym_half<0>(src, atab[jb]);
                        } else {
                            o = (e & 1) ? sm_half_to_e4m3_fast<4>(src) : sm_half_to_e4m3_fast<0>(src);
                        }
                        keep_here(o);
                        next.op[jb][e] = (int)o;
                    }
                    p_prev = p;
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);              // LDS reads of the next block
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);              // this step's MFMA
                    __builtin_amdgcn_sched_group_barrier(0x002, (IN_MFMA ? 0 : 4) + (ASYM ? 7 : 4) * PIECES, 0);   // ALU work independent of it
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (!IN_MFMA) {
                const float sc = fabsf(cur.s[TPW - 1]);
                acc[MF - 1][TPW - 1][0] = fmaf(sc, p_prev[0], acc[MF - 1][TPW - 1][0]);
                acc[MF - 1][TPW - 1][1] = fmaf(sc, p_prev[1], acc[MF - 1][TPW - 1][1]);
                acc[MF - 1][TPW - 1][2] = fmaf(sc, p_prev[2], acc[MF - 1][TPW - 1][2]);
                acc[MF - 1][TPW - 1][3] = fmaf(sc, p_prev[3], acc[MF - 1][TPW - 1][3]);
            }
            // The -8 fix-up of the freshly expanded operand, for the bands whose next chunk is marked: here, after the
            // steps, so that the step sequence above stays one basic block (a wave-uniform branch per piece of the
            // expansion would cut it up, and the order of MFMAs, LDS reads and ALU work cannot be held across blocks).
            if (!ASYM) {
#pragma unroll
                for (int j = 0; j < TPW; ++j) {
                    if (m8[j]) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const int d = e >> 1;
                            const uint32_t src = d == 0 ? raw[j].x : d == 1 ? raw[j].y : d == 2 ? raw[j].z : raw[j].w;
                            const uint32_t o = (uint32_t)next.op[j][e];
                            next.op[j][e] = TWO ? (int)((e & 1) ? two_level_fix_minus_eight<4>(o, src, tab[j])
                                                                : two_level_fix_minus_eight<0>(o, src, tab[j]))
                                                : (int)sm_fix_minus_eight(o);
                        }
                    }
                }
            }
        }
        __builtin_amdgcn_s_setprio(0);
        lds_dma_wait_all();                                      // this wavefront's copies have landed ...
        __syncthreads();                                         // ... and so have everyone's; the block just read is free
    };

    Band wa, wb;
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        wa.op[j] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
        wb.op[j] = wa.op[j];
        wa.s[j] = 0.f;
        wb.s[j] = 0.f;
    }
    {
        // the group's first chunk comes through registers, so that the copies of its second chunk need not wait for it
        uint4 raw0[TPW];
        uint32_t zp0[TPW];
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
            raw0[j] = make_uint4(0u, 0u, 0u, 0u);
            zp0[j] = 0u;
            if (kg < C) {
                raw0[j] = *reinterpret_cast<const uint4*>(wbase[j] + (int64_t)kg * 1024 + woff);
                wa.s[j] = *reinterpret_cast<const float*>(sbase[j] + (int64_t)(kg / cpg) * REC + soff);
                if (ASYM) zp0[j] = sbase[j][(int64_t)(kg / cpg) * REC + 64 + i];
            }
        }
        stage_x(0, 0);
        if (kg + KS < C) stage_w(kg + KS, 0u);
#pragma unroll
        for (int j = 0; j < TPW; ++j)
            wa.op[j] = TWO    ? slot_to_operand_two_level<true>(raw0[j], two_level_table(wa.s[j]))
                       : ASYM2 ? slot_to_operand_asym(raw0[j], asym_two_level_table(zp0[j], wa.s[j]))
                       : ASYM  ? slot_to_operand_asym(raw0[j], asym_table(zp0[j]))
                              : slot_to_operand<true>(raw0[j]);
    }
    lds_dma_wait_all();
    __syncthreads();

    for (int ps = 0; ps < passes; ps += 2) {
        pass(ps, wa, wb);                                        // even pass: A multiplies, the next chunk expands into B
        if (ps + 1 < passes) pass(ps + 1, wb, wa);
    }

    // K-split groups 1 .. KS-1 hand their partial sums to group 0 through LDS (the loop's last barrier has passed:
    // nobody reads activations any more).
    if (KS > 1) {
        float* red = reinterpret_cast<float*>(lds);
        if (kg > 0) {
#pragma unroll
            for (int f = 0; f < MF; ++f)
#pragma unroll
                for (int j = 0; j < TPW; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        red[(((((kg - 1) * NB + band) * MF + f) * TPW + j) * 4 + r) * 64 + lane] = acc[f][j][r];
        }
        __syncthreads();
        if (kg == 0) {
#pragma unroll
            for (int k2 = 1; k2 < KS; ++k2)
#pragma unroll
                for (int f = 0; f < MF; ++f)
#pragma unroll
                    for (int j = 0; j < TPW; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            acc[f][j][r] += red[(((((k2 - 1) * NB + band) * MF + f) * TPW + j) * 4 + r) * 64 + lane];
        }
        __syncthreads();
    }

    // Epilogue.  Result lane: channel = lane % 16 of the band, tokens 4*kq .. 4*kq+3 of block f.  The workgroup turns
    // FR 16-token slabs at a time into row-major order in LDS and stores whole BN-channel row segments.
    const float sx = *s_x;
    const float yq = (sizeof(OutT) == 1) ? *y_scale : 1.0f;      // FP8 output: the next layer's activation scale
    float so[TPW];                                               // output scale of the lane's channel of each band
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        const int n = bn * BN + (band * TPW + j) * 16 + i;
        so[j] = OUT_SCALED ? sx * w_out[per_channel ? min(n, N - 1) : 0] : sx;
    }
    SlabT* slab = reinterpret_cast<SlabT*>(lds);
    constexpr int VEC = SILU ? 16 : 16 / sizeof(SlabT);          // outputs per 16-byte store
    constexpr int UPR = (SILU ? BN / 2 : BN) / VEC;              // 16-byte units per row
    const int n_block = bn * BN;
    const bool vec_ok = (ldy % VEC == 0) && (reinterpret_cast<uintptr_t>(y) % 16 == 0);
#pragma unroll
    for (int f0 = 0; f0 < MF; f0 += FR) {
        if (kg == 0) {
#pragma unroll
            for (int ff = 0; ff < FR; ++ff) {
                if (f0 + ff < MF) {
#pragma unroll
                    for (int j = 0; j < TPW; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            slab[(ff * 16 + 4 * kq + r) * RS + (band * TPW + j) * 16 + i] =
                                OutCast<SlabT>::cast(so[j] * acc[(f0 + ff < MF) ? f0 + ff : 0][j][r], yq);
                }
            }
        }
        __syncthreads();
        constexpr int ROWS = FR * 16;
        for (int u = tid; u < ROWS * UPR; u += WAVES * 64) {
            const int row = u / UPR, col = (u % UPR) * VEC;
            const int m = m0 + f0 * 16 + row;
            if constexpr (SILU) {
                // 16 outputs of one band pair: gate = slab columns 32p .. 32p+15, up = 32p+16 .. 32p+31 (p = col / 16)
                const int n_out = n_block / 2 + col;             // first of the 16 output columns; N / 2 columns in all
                if (row < (MF - f0) * 16 && m < M && n_out < N / 2) {
                    const SlabT* g = slab + row * RS + 2 * col;
                    uint8_t* dst = reinterpret_cast<uint8_t*>(y) + (int64_t)m * ldy + n_out;
                    uint32_t w[4];
#pragma unroll
                    for (int e = 0; e < 16; e += 4) {
                        float h[4];
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            h[t] = bf16_bits_to_f32(f32_to_bf16_bits(
                                silu_mul_f32(bf16_bits_to_f32(g[e + t]), bf16_bits_to_f32(g[16 + e + t]))));
                        w[e / 4] = cvt2(h[2] / yq, h[3] / yq, cvt2(h[0] / yq, h[1] / yq, 0u, false), true);
                    }
                    if (vec_ok && n_out + 16 <= N / 2) {
                        *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
                    } else {
                        for (int e = 0; e < 16 && n_out + e < N / 2; ++e) dst[e] = (uint8_t)(w[e / 4] >> (8 * (e % 4)));
                    }
                }
            } else {
                const int n = n_block + col;
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
        }
        __syncthreads();
    }
}

template <typename OutT, int MF, int KS, int TPW>
void launch_one(const LinearArgs& a, dim3 grid, int grid_m, int grid_n, hipStream_t st) {
#define W4A8_MFMA(MODEV)                                                                                                   \
    hipLaunchKernelGGL((linear_mfma_kernel<OutT, MF, KS, TPW, MODEV>), grid, dim3(WAVES * 64), 0, st, a.x8, a.M, a.ldx8, a.s_x, \
                       a.packed, a.scales, a.N, a.n_tiles, a.C, a.cpg, a.NG, static_cast<OutT*>(a.y), a.ldy, grid_m, grid_n,   \
                       a.w_out, a.per_channel, a.y_scale)
    if constexpr (sizeof(OutT) == 1) {                           // FP8 output exists for the code-exact mode only
        W4A8_MFMA(MODE_CODE_EXACT);
        return;
    } else {
    if (a.mode == MODE_TWO_LEVEL)
        W4A8_MFMA(MODE_TWO_LEVEL);
    else if (a.mode == MODE_ASYM)
        W4A8_MFMA(MODE_ASYM);
    else if (a.mode == MODE_POW2)
        W4A8_MFMA(MODE_POW2);
    else if (a.mode == MODE_ASYM_TWO)
        W4A8_MFMA(MODE_ASYM_TWO);
    else
        W4A8_MFMA(MODE_CODE_EXACT);
    }
#undef W4A8_MFMA
}

}  // namespace

// Launch shape of the many-token kernels for a layer; requested values of mf / ks / tpw other than 0 are kept.
// cfg2d >= 0 on return: the layer goes to the second tiling (linear_mfma2d.hip) with that workgroup tile.
//  - In the code-exact and power-of-two modes the second tiling (a 2-D grid of wavefronts over 256-token tiles,
//    expansion shared through LDS, persistent workgroups) competes with the first on estimated time.  A persistent
//    workgroup needs a fixed time per tile, so what a grid costs is rounds x time per tile, and the last, partly filled
//    round costs as much as a full one: 256 x 256 tiles (one workgroup per compute unit, 256 at a time), 256 x 128 tiles
//    with eight wavefronts (256 at a time) or with four (two workgroups per compute unit, 512 at a time; a tile takes
//    longer while two share the unit).  Times per tile in microseconds, C = K / 128 chunks, from medians on the
//    Llama-3 layer shapes with the weights coming from HBM: 6 + 1.66 C, 5 + 1.08 C, 5 + 1.28 C alone and 5 + 1.875 C
//    shared (half of that for a last round of at most 256 tiles that follows full ones).  The first tiling is priced
//    at 0.265 C + flops / 1.35 PFLOP/s.  Against the rule this replaces (256 x 256 or
//    four-wavefront 256 x 128 tiles once they number 200): 640 tokens on gate|up 125 -> 104 us, 3072 / 4096 tokens on
//    QKV 113 / 120 -> 101 / 108, 2048 tokens on the O projection 47 -> 42, 192...256 tokens on gate|up 48 -> 42.
//  - First tiling: tall token blocks amortize the nibble expansion over more MFMAs; two bands per wavefront halve the
//    LDS reads per MFMA (the activation operand is reused); K-splits shorten the dependent chain of passes (each waits
//    for the copies of the next) when the grid is too small to fill the chip, at the price of a wider activation block
//    to copy per pass.  Sweeps over the Llama-3 layer shapes are matched by: the first shape, in the list's order of
//    preference, that yields about 1.5 workgroups per compute unit.
bool mfma_launch_shape(int64_t M, int64_t K, int64_t N, int mode, int& mf, int& ks, int& tpw, int& cfg2d) {
    cfg2d = -1;
    const int C = (int)(K / 128);
    const int n_tiles = (int)((N + 15) / 16);
    if (mf == 0 && ks == 0 && tpw == 0 && (mode == MODE_CODE_EXACT || mode == MODE_POW2 || mode == MODE_TWO_LEVEL)) {
        const int64_t tm = (M + 255) / 256, t1 = tm * ((N + 255) / 256), t2 = tm * ((N + 127) / 128);
        const double c = (double)C;
        const double e1 = (double)((t1 + 255) / 256) * (6.0 + 1.66 * c);
        const double e2 = (double)((t2 + 255) / 256) * (5.0 + 1.08 * c);
        const int64_t full = t2 / 512, rem = t2 % 512;
        const double shared = 5.0 + 1.875 * c;                   // a tile while two workgroups share the compute unit
        // the last, partly filled round: alone on their units the workgroups run faster, and after full rounds they start
        // it while others still finish theirs (measured: about half a shared round then)
        const double e4 = (double)full * shared + (rem == 0 ? 0.0 : rem > 256 ? shared : full > 0 ? 0.5 * shared : 5.0 + 1.28 * c);
        const double first = 0.265 * c + 2.0 * (double)M * (double)K * (double)N / 1.35e9;
        const double best = e1 < e2 ? (e1 < e4 ? e1 : e4) : (e2 < e4 ? e2 : e4);
        if (best < first) {
            cfg2d = best == e1 ? 1 : best == e2 ? 2 : 4;
            return true;
        }
    }
    static const int cand[W4A8_MFMA_SHAPES][3] = W4A8_MFMA_SHAPE_LIST;
    if (mf == 0 || ks == 0 || tpw == 0) {
        int pick = -1, fallback = -1;
        // 256 tokens x 256 channels (two bands per wavefront, half the LDS reads per MFMA, one workgroup per compute unit)
        // measured no faster than 256 x 128 at twice the occupancy on any swept shape: on request only.
        if (tpw == 2 && (mf == 0 || mf == 16) && (ks == 0 || ks == 1)) pick = W4A8_MFMA_SHAPES - 1;
        for (int q = 0; q < W4A8_MFMA_SHAPES - 1 && pick < 0; ++q) {
            const int mfv = cand[q][0], ksv = cand[q][1], tpv = cand[q][2];
            if ((mf && mf != mfv) || (ks && ks != ksv) || (tpw && tpw != tpv)) continue;
            fallback = q;                                        // the finest shape that matches the request
            if (mfv > 4 && 16 * mfv >= 2 * M + 64) continue;     // mostly padding
            if (ksv > 1 && C < 4 * ksv) continue;                // too few chunks to split
            const int per_wg = (8 / ksv) * tpv;
            const int64_t groups = ((M + 16 * mfv - 1) / (16 * mfv)) * (int64_t)((n_tiles + per_wg - 1) / per_wg);
            if (groups >= 384) { pick = q; break; }
        }
        if (pick < 0) pick = fallback;
        if (pick < 0) return false;                              // a combination that is not built
        mf = cand[pick][0];
        ks = cand[pick][1];
        tpw = cand[pick][2];
    }
    return true;
}

// mf = 16-token blocks per workgroup (4, 8 or 16), ks = K-split groups (1, 2 or 4), tpw = weight bands per wavefront
// (1 or 2); 0 = chosen from the shape.
int launch_linear_mfma_tiled(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x,
                             const uint8_t* packed, const float* scales, int64_t N, int32_t G, void* y,
                             w4a8_dtype ydt, int64_t ldy, int mf, int ks, int tpw, const float* w_out, int per_channel,
                             int mode, const float* y_scale, hipStream_t st) {
    if (((int)ydt == YDT_E4M3 || (int)ydt == YDT_SILU_E4M3) && (mode != MODE_CODE_EXACT || !y_scale)) return W4A8_ERR_DTYPE;
    if ((int)ydt == YDT_SILU_E4M3 && N % 32 != 0) return W4A8_ERR_SHAPE;   // whole pairs of gate and up bands
    if (!(mf == 0 || mf == 4 || mf == 8 || mf == 16) || !(ks == 0 || ks == 1 || ks == 2 || ks == 4) || tpw < 0 || tpw > 2)
        return W4A8_ERR_SHAPE;
    const int C = (int)(K / 128), cpg = G / 128, NG = (int)(K / G);
    const int n_tiles = (int)((N + 15) / 16);
    int cfg2d = -1;
    if (!mfma_launch_shape(M, K, N, mode, mf, ks, tpw, cfg2d)) return W4A8_ERR_SHAPE;
    if (cfg2d >= 0)
        return launch_linear_mfma2d(x8, M, K, ldx8, s_x, packed, scales, N, G, y, ydt, ldy, cfg2d, 0, 0, mode, y_scale, st, 1, nullptr,
                                    w_out, per_channel);
    const int per_wg = (8 / ks) * tpw;
    const int grid_n = (n_tiles + per_wg - 1) / per_wg;
    const int grid_m = (int)((M + 16 * mf - 1) / (16 * mf));
    const int64_t total = (int64_t)grid_m * grid_n;
    if (total > (1 << 30)) return W4A8_ERR_SHAPE;
    if (ldx8 >= (1 << 24)) return W4A8_ERR_SHAPE;               // 32-bit activation offsets inside a token block
    const dim3 grid((unsigned)((total + XCDS - 1) / XCDS * XCDS));
    const LinearArgs a{x8, (int)M, ldx8, s_x, packed, scales, (int)N, n_tiles, C, cpg, NG, y, ldy, w_out, per_channel, mode, y_scale};
    bool launched = false;
#define W4A8_CASE(MFV, KSV, TPV)                                              \
    if (mf == MFV && ks == KSV && tpw == TPV) {                               \
        launched = true;                                                      \
        if (ydt == W4A8_F32)                                                  \
            launch_one<float, MFV, KSV, TPV>(a, grid, grid_m, grid_n, st);    \
        else if ((int)ydt == YDT_SILU_E4M3)                                   \
            launch_one<SiluFp8, MFV, KSV, TPV>(a, grid, grid_m, grid_n, st);  \
        else if ((int)ydt == YDT_E4M3)                                        \
            launch_one<uint8_t, MFV, KSV, TPV>(a, grid, grid_m, grid_n, st);  \
        else                                                                  \
            launch_one<uint16_t, MFV, KSV, TPV>(a, grid, grid_m, grid_n, st); \
    }
    W4A8_CASE(16, 1, 2) W4A8_CASE(16, 1, 1) W4A8_CASE(8, 1, 1) W4A8_CASE(8, 2, 1) W4A8_CASE(4, 1, 1)
    W4A8_CASE(4, 2, 1) W4A8_CASE(4, 4, 1)
#undef W4A8_CASE
    if (!launched) return W4A8_ERR_SHAPE;
    return launch_status();
}

}  // namespace w4a8
