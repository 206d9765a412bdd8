// W4A8 linear layer for many tokens, second tiling: a two-dimensional grid of wavefronts over a large workgroup tile, with
// the INT4 -> E4M3 expansion (Eq. 10) done ONCE per workgroup and weight band and shared through LDS, in persistent
// workgroups that walk over the output tiles.
//
// A workgroup of eight wavefronts, arranged WGM (tokens) x WGN (channels), computes BM = 16*WM*WGM tokens x
// BN = 16*WN*WGN channels of Y per tile; a wavefront owns WM 16-token blocks x WN 16-channel bands.  Per 128-deep chunk:
//   - the activation block (BM x 128 bytes) travels global -> LDS without passing through registers (lds_dma_16), one
//     chunk ahead, double buffered; the copy instructions are spread over the MFMA steps of the first half of a chunk
//     (issued in a burst at its head they hold the vector memory path while every matrix unit of the compute unit idles);
//   - every wavefront expands EPW = WN / WGM of the workgroup's weight bands for the NEXT chunk (raw nibbles loaded into
//     registers one chunk earlier still) and publishes the finished E4M3 operand in LDS in operand order (lane-linear
//     16-byte accesses, free of bank conflicts); all WGM wavefronts that multiply with that band read it from there.
//     The expansion therefore costs 32 ALU operations per band and chunk for the whole BM-token tile, where a wavefront
//     that expands its own band pays them per 16 * WM tokens;
//   - a wavefront keeps its WN weight operands in registers for the chunk and streams its WM activation operands through
//     them: one LDS operand read feeds WN MFMAs;
//   - weights are the column operand of the 16x16x128 MFMA, so a result lane holds one channel and its group scale is a
//     single register: each MFMA starts from a zero accumulator and is folded into the running sum with four FMAs
//     (Eq. 10 with the scale factored out of the group's sum), two steps later, when its result has long arrived; for
//     power-of-two scales the matrix unit applies the scale itself and the sum stays in its accumulator;
//   - one workgroup barrier per chunk.  Register-destination loads of a chunk (group scales, raw nibbles) are issued at
//     its head and first touched right after the next barrier, when the wavefront has waited for all of its loads
//     anyway, so that the compiler's own wait counts (which do not see the LDS copies) never ask for a load that was
//     only just issued.  The nibbles travel as one 128-bit value: split into four, the register allocator moved parts of
//     it right after the load, which waits for the load on the spot.
// What bounds the loop is instruction issue: a SIMD's vector port is taken for about 16 cycles by an MFMA and 4 by any
// other vector instruction, so 32 cycles of matrix work leave room for four of those -- the four FMAs; every further
// instruction per MFMA (the expansion: 2 at 256 tokens per tile, 1 at 512) shows in the rate.
// Tiles: a workgroup is resident for the whole launch and takes every (workgroups per XCD)-th tile of its XCD's
// contiguous share of a block order that walks group_m token blocks per channel block, so the tiles an XCD works on at
// a time cover a compact rectangle (one L2 per XCD).  The first loads and copies of the NEXT tile are issued before
// the epilogue of the current one and finished in its middle: a tile's cold start (two memory round trips) is hidden.
// Epilogue for float32 / bf16 outputs: straight from the accumulators -- neighbouring lanes exchange two of their four
// tokens (DPP), so that a lane holds two adjacent channels of two tokens, converted by the hardware's bf16 conversion
// and stored as 4-byte pieces; the four bands of a wavefront complete 128-byte lines.  No LDS, no barriers.
// The -8 pattern of the sign-magnitude nibbles comes out of the fast expansion as minus zero; the wavefronts that read a
// band put it right in their registers on chunks whose group scale carries the packer's mark.
#include "w4a8_device.hpp"
#include "w4a8_internal.hpp"

#include <math.h>

#include <utility>

namespace w4a8 {
namespace {

constexpr int XCDS2 = 8;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order: an unrolled loop whose index is a constant
// expression inside the body (the scheduling builtins take constants only).
template <int... I, typename F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, I...>, F&& f) {
    (f(std::integral_constant<int, I>{}), ...);
}

// A wave-uniform pointer, marked as such: a load from `uniform(p) + lane_offset` (32-bit offset) then takes its base from
// scalar registers instead of a 64-bit address per lane that the compiler would keep, and advance, in vector registers.
#define W4A8_GLOBAL __attribute__((address_space(1)))
__device__ __forceinline__ const W4A8_GLOBAL uint8_t* uniform(const uint8_t* p) {
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    return reinterpret_cast<const W4A8_GLOBAL uint8_t*>(((uint64_t)hi << 32) | lo);
}

// the value of the neighbouring lane (lane ^ 1)
__device__ __forceinline__ uint32_t from_pair_lane(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1 /* quad_perm [1, 0, 3, 2] */, 0xF, 0xF, true);
}

template <typename OutT, int WGM, int WGN, int WM, int WN, int MODE>
__global__ void __launch_bounds__(64 * WGM * WGN, 2) linear_mfma2d_kernel(
    const uint8_t* __restrict__ x8, int M, int64_t ldx8, const float* __restrict__ s_x,
    const uint8_t* __restrict__ packed, const float* __restrict__ scales, int N, int n_tiles, int C, int cpg, int NG,
    OutT* __restrict__ y, int64_t ldy, int grid_m, int grid_n, int group_m, const float* __restrict__ y_scale, int ksplit,
    int cps, int64_t split_stride, const float* __restrict__ w_out, int per_channel) {
    constexpr int WAVES = WGM * WGN, THREADS = 64 * WAVES;
    static_assert(WAVES == 8 || WAVES == 4, "one workgroup of eight wavefronts per compute unit, or two of four");
    static_assert(WN % WGM == 0, "every wavefront expands whole bands of its own");
    // Eight wavefronts own the compute unit's LDS (160 KB) and keep two stages of weight operands.  Four leave half of
    // it to a second workgroup on the same compute unit, whose chunks drift against this one's, so that one's barriers
    // and operand reads at the head of a chunk fall into the other's MFMA steps; they keep ONE stage of weight operands,
    // which costs a second barrier per chunk (all operand registers read before the next chunk's operands are written).
    constexpr int B_STAGES = WAVES == 8 ? 2 : 1;
    static_assert(MODE == MODE_CODE_EXACT || MODE == MODE_POW2 || MODE == MODE_TWO_LEVEL, "modes built for this tiling");
    constexpr bool POW2 = MODE == MODE_POW2;
    // Two-level reading (Eq. 6-11 taken literally): `scales` are FP8-domain group scales, the weight operand is
    // nearest_E4M3(code * s8[n, g]) -- formed by the wavefront that expands the band, which therefore loads the scales of
    // the bands it expands, not of those it multiplies with -- the sum over all of K stays in the matrix unit and the
    // output is scaled by s_x * w_out[n] (w_out[0] when per_channel is 0).
    constexpr bool TWO = MODE == MODE_TWO_LEVEL;
    constexpr bool SUM_IN_MFMA = POW2 || TWO;                    // no FMAs in the loop
    constexpr int BM = 16 * WM * WGM, BN = 16 * WN * WGN;
    constexpr int NBAND = WN * WGN;                              // weight bands of the workgroup tile
    constexpr int EPW = WN / WGM;                                // bands a wavefront expands per chunk
    constexpr int A_STAGE = BM * 128, B_STAGE = NBAND * 2048;
    constexpr int STAGE = A_STAGE + (B_STAGES == 2 ? B_STAGE : 0);   // activation stage s at s * STAGE, its weight operands behind it
    constexpr int B_OFF = B_STAGES == 2 ? A_STAGE : 2 * A_STAGE;     // the single stage of weight operands: behind both activation stages
    constexpr int DPW = BM / (8 * WAVES);                        // 1 KiB activation pages a wavefront copies per chunk
    static_assert(DPW % 2 == 0, "a wavefront copies whole 16-token blocks");
    constexpr int LOOP_BYTES = 2 * STAGE + (B_STAGES == 2 ? 0 : B_STAGE);
    using SlabT = typename OutKind<OutT>::Slab;
    constexpr bool SILU = OutKind<OutT>::SILU;
    constexpr bool DIRECT = !SILU && sizeof(OutT) >= 2;          // float32 / bf16: stored from the accumulators
    constexpr int RS = BN + 16 / sizeof(SlabT);                  // slab epilogue: row stride, rows stay 16-byte aligned
    constexpr int SLAB_ROWS = 16 * WGM;                          // one 16-token block of every wavefront row per round
    static_assert(DIRECT || SLAB_ROWS * RS * (int)sizeof(SlabT) <= (B_STAGES == 2 ? STAGE : A_STAGE), "the epilogue slab fits stage 1");
    constexpr int STEPS = WM * WN;                               // MFMAs per chunk and wavefront
    static_assert((8 * EPW) <= STEPS && STEPS % (8 * EPW) == 0, "an eighth of the expansion every few steps");
    constexpr int STEPS_PER_EIGHTH = STEPS / (8 * EPW);
    constexpr int DMA_EVERY = (STEPS / 2) / DPW > 0 ? (STEPS / 2) / DPW : 1;   // steps between two activation copies
    static_assert(DMA_EVERY * DPW <= STEPS, "the copies fit the chunk");
    __shared__ __attribute__((aligned(16))) uint8_t lds[LOOP_BYTES];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int kq = lane >> 4, i = lane & 15;

    // This workgroup's tiles: consecutive workgroup ids go round-robin to the eight XCDs; XCD x owns the contiguous range
    // [x * per_xcd, (x + 1) * per_xcd) of the virtual tile order, and its workgroups take every nx-th tile of it.
    // With ksplit > 1 a unit of work is (K range, tile): unit u multiplies chunks [u / tiles * cps, + cps) of tile
    // u % tiles and stores its float32 partial sums, unscaled, at y + (u / tiles) * split_stride (the workspace).
    const int tiles = grid_m * grid_n;
    const int total = tiles * ksplit;
    const int nx = gridDim.x / XCDS2;
    const int per_xcd = (total + XCDS2 - 1) / XCDS2;
    const int v_end = min(total, (int)(blockIdx.x % XCDS2 + 1) * per_xcd);
    int v = (int)(blockIdx.x % XCDS2) * per_xcd + (int)(blockIdx.x / XCDS2);
    if (v >= v_end) return;

    // state of the unit whose loads are being issued (the main loop's unit)
    int m0 = 0, bn = 0, split = 0, c_begin = 0, c_end = C;
    const uint8_t* sbase[WN];                                    // scales of the wavefront's bands: + g * 64 + i * 4
    const uint8_t* ebase[EPW];                                   // nibbles of the bands it expands: + c * 1024 + lane * 16
    const uint8_t* esbase[EPW];                                  // two-level mode: their scales, + g * 64 + i * 4
    const uint8_t* xrow0 = x8;
    uint32_t xoff[DPW];                                          // lane's offset of page q from the tile's first row
    const uint32_t woff = lane * 16, soff = i * 4;
    // Activation stage in LDS: 16-token block b = 2 KiB = two 1 KiB pages of 8 rows x 128 bytes; 16-byte segment sg of
    // row r (0..15) sits in page r / 8 at slot (r % 8) * 8 + (sg ^ (r % 8) ^ (r / 8)): one copy instruction fills a
    // page from eight whole 128-byte row segments, and the two ds_read_b128 of an operand are free of bank conflicts.
    // A wavefront copies pages wave * DPW .. + DPW - 1; page d holds rows 8 (d % 2) .. + 7 of block d / 2.
    auto set_tile = [&](int unit) {
        split = unit / tiles;
        const int vt = unit - split * tiles;
        c_begin = split * cps;
        c_end = min(C, c_begin + cps);
        const int group = vt / (group_m * grid_n);
        const int first_m = group * group_m;
        const int rows_in_group = min(group_m, grid_m - first_m);
        const int in_group = vt - group * group_m * grid_n;
        const int bm = first_m + in_group % rows_in_group;
        bn = in_group / rows_in_group;
        m0 = bm * BM;
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int t = min(bn * NBAND + wn * WN + j, n_tiles - 1);   // bands past the end reload the last one; not stored
            sbase[j] = reinterpret_cast<const uint8_t*>(scales) + (int64_t)t * NG * 64;
        }
#pragma unroll
        for (int t = 0; t < EPW; ++t) {
            const int tt = min(bn * NBAND + wn * WN + wm * EPW + t, n_tiles - 1);
            ebase[t] = packed + (int64_t)tt * C * 1024;
            esbase[t] = reinterpret_cast<const uint8_t*>(scales) + (int64_t)tt * NG * 64;
        }
        xrow0 = x8 + (int64_t)m0 * ldx8;
#pragma unroll
        for (int q = 0; q < DPW; ++q) {
            const int r = (q & 1) * 8 + (lane >> 3);
            const int row = min(m0 + (wave * (DPW / 2) + q / 2) * 16 + r, M - 1) - m0;   // rows past the end reload the last row; not stored
            xoff[q] = (uint32_t)row * (uint32_t)ldx8 + (uint32_t)(((lane & 7) ^ (r & 7) ^ (r >> 3)) * 16);
        }
    };
    const uint32_t xa_off = (uint32_t)((wm * WM) * 2048 + (i >> 3) * 1024 + ((i & 7) * 8 + ((2 * kq) ^ ((i & 7) ^ (i >> 3)))) * 16);
    const uint32_t xc_off = (uint32_t)((wm * WM) * 2048 + (i >> 3) * 1024 + ((i & 7) * 8 + ((2 * kq + 1) ^ ((i & 7) ^ (i >> 3)))) * 16);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;
    uint8_t* const b_lds = lds + B_OFF;                          // + (stage * STAGE) + band * 2048 + half * 1024 + lane * 16

    // page q of this wavefront's share of chunk c's activations into stage `buf`
    auto stage_page = [&](int c, int buf, int q) {
        lds_dma_16(xrow0 + (int64_t)c * 128, xoff[q], lds0 + (uint32_t)buf * STAGE + (uint32_t)wave * (DPW * 1024) + q * 1024);
    };

    struct Set {
        float s[WN];                                             // group scales of the wavefront's bands
        u32x4 raw[EPW];                                          // nibbles of the bands it expands, one chunk further on
        float es[EPW];                                           // two-level mode: the group scales that go with them
    };
    auto load_scales = [&](Set& S, int c) {
        if (TWO) return;                                         // the multiplying wavefronts need no scales there
#pragma unroll
        for (int j = 0; j < WN; ++j) S.s[j] = *reinterpret_cast<const W4A8_GLOBAL float*>(uniform(sbase[j] + (int64_t)(c / cpg) * 64) + soff);
    };
    auto load_raw = [&](Set& S, int c) {
#pragma unroll
        for (int t = 0; t < EPW; ++t) S.raw[t] = *reinterpret_cast<const W4A8_GLOBAL u32x4*>(uniform(ebase[t] + (int64_t)c * 1024) + woff);
        if (TWO) {
#pragma unroll
            for (int t = 0; t < EPW; ++t) S.es[t] = *reinterpret_cast<const W4A8_GLOBAL float*>(uniform(esbase[t] + (int64_t)(c / cpg) * 64) + soff);
        }
    };
    // the finished operand of expanded band t (registers 4h .. 4h+3) into stage `buf`
    auto publish = [&](int buf, int t, int h, uint32_t a, uint32_t b, uint32_t c2, uint32_t d) {
        uint8_t* dst = b_lds + (B_STAGES == 2 ? buf * STAGE : 0) + (wn * WN + wm * EPW + t) * 2048 + h * 1024 + lane * 16;
        *reinterpret_cast<uint4*>(dst) = make_uint4(a, b, c2, d);
    };

    v4f acc[WM][WN];

    // One chunk: multiply chunk c (activations and weight operands in stage c % 2) with the scales cur.s; meanwhile
    // expand cur.raw (chunk c + 1) into the other stage, copy the activations of chunk c + 1 there, and load the scales
    // of chunk c + 1 and the nibbles of chunk c + 2 into nxt.
    auto chunk = [&](int c, Set& cur, Set& nxt) {
        const int buf = (c - c_begin) & 1;
        // what the previous chunk loaded is touched here, straight after the wait for all loads at that chunk's end
        if (!TWO) {
#pragma unroll
            for (int j = 0; j < WN; ++j) asm volatile("" : "+v"(cur.s[j]));
        }
#pragma unroll
        for (int t = 0; t < EPW; ++t) asm volatile("" : "+v"(cur.raw[t]));   // as one 128-bit value: it stays in the registers it was loaded into
        MagTable tab[EPW];                                       // two-level mode: nearest_E4M3(m * s8) for the lane's channel
        if (TWO) {
#pragma unroll
            for (int t = 0; t < EPW; ++t) {
                asm volatile("" : "+v"(cur.es[t]));
                tab[t] = two_level_table(cur.es[t]);
            }
        }
        const int cn = min(c + 1, c_end - 1);                    // after the last chunk: copied again, never read
        if (c + 1 < c_end) load_scales(nxt, c + 1);
        if (c + 2 < c_end) load_raw(nxt, c + 2);

        __builtin_amdgcn_s_setprio(1);
        // the wavefront's weight operands of this chunk
        v8i bop[WN];
        const uint8_t* bsrc = b_lds + (B_STAGES == 2 ? buf * STAGE : 0) + (wn * WN) * 2048 + lane * 16;
        const uint8_t* xb = lds + buf * STAGE;
        uint4 xa = *reinterpret_cast<const uint4*>(xb + xa_off);
        uint4 xc = *reinterpret_cast<const uint4*>(xb + xc_off);
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const uint4 lo = *reinterpret_cast<const uint4*>(bsrc + j * 2048);
            const uint4 hi = *reinterpret_cast<const uint4*>(bsrc + j * 2048 + 1024);
            bop[j] = v8i{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
        }
        if (B_STAGES == 1) {
            // one stage of weight operands: everybody's operand registers are filled before anybody publishes the next chunk's
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __syncthreads();
        }
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            if (!TWO && any_marked(cur.s[j])) {                  // wave-uniform, rare: the band's group holds a -8
#pragma unroll
                for (int e = 0; e < 8; ++e) bop[j][e] = (int)sm_fix_minus_eight((uint32_t)bop[j][e]);
            }
        }
        uint32_t eop[EPW][8];
        // products of the last two steps: a step folds in the one before last, whose MFMA has long finished
        v4f p_prev = v4f{0.f, 0.f, 0.f, 0.f}, p_prev2 = v4f{0.f, 0.f, 0.f, 0.f};
        auto fold = [&](auto FP, auto JP, const v4f& p) {
            constexpr int fp = decltype(FP)::value, jp = decltype(JP)::value;
            const float sc = fabsf(cur.s[jp]);                   // the sign bit is the packer's mark, not part of the scale
            acc[fp][jp][0] = fmaf(sc, p[0], acc[fp][jp][0]);
            acc[fp][jp][1] = fmaf(sc, p[1], acc[fp][jp][1]);
            acc[fp][jp][2] = fmaf(sc, p[2], acc[fp][jp][2]);
            acc[fp][jp][3] = fmaf(sc, p[3], acc[fp][jp][3]);
        };
        v8i xop = v8i{0, 0, 0, 0, 0, 0, 0, 0};
        static_for(std::make_integer_sequence<int, STEPS>{}, [&](auto ST) {
            constexpr int st = decltype(ST)::value, f = st / WN, j = st % WN;
            if (j == 0) {
                xop = v8i{(int)xa.x, (int)xa.y, (int)xa.z, (int)xa.w, (int)xc.x, (int)xc.y, (int)xc.z, (int)xc.w};
                if (f + 1 < WM) {
                    xa = *reinterpret_cast<const uint4*>(xb + xa_off + (f + 1) * 2048);
                    xc = *reinterpret_cast<const uint4*>(xb + xc_off + (f + 1) * 2048);
                }
            }
            // the copies of the next chunk's activations, one every few steps of the first half of the chunk
            if constexpr (st % DMA_EVERY == 0 && st / DMA_EVERY < DPW) stage_page(cn, buf ^ 1, st / DMA_EVERY);
            if (POW2) acc[f][j] = mfma_16x16x128_e4m3_scaled(xop, bop[j], acc[f][j], E8M0_ONE, e8m0_of(cur.s[j]));
            if (TWO) acc[f][j] = mfma_16x16x128_e4m3(xop, bop[j], acc[f][j]);
            const v4f p = SUM_IN_MFMA ? v4f{0.f, 0.f, 0.f, 0.f} : mfma_16x16x128_e4m3(xop, bop[j], v4f{0.f, 0.f, 0.f, 0.f});
            if constexpr (!SUM_IN_MFMA && st > 1) {
                fold(std::integral_constant<int, (st - 2) / WN>{}, std::integral_constant<int, (st - 2) % WN>{}, p_prev2);
                keep_here(acc[(st - 2) / WN][(st - 2) % WN]);
            }
            p_prev2 = p_prev;
            p_prev = p;
            // this step's share of the next chunk's expansion: eighth E of the EPW bands is operand register E % 8 of
            // band E / 8 (half E % 2 of dword (E % 8) / 2); a finished half of an operand goes to LDS at once
            // (also in the last chunk, where nobody reads the result: a branch here would cut the step sequence up)
            constexpr bool EXPAND = st % STEPS_PER_EIGHTH == STEPS_PER_EIGHTH - 1;
            constexpr int E = st / STEPS_PER_EIGHTH, t = E / 8, e = E % 8, d = e >> 1;
            if constexpr (EXPAND) {
                const uint32_t src = cur.raw[t][d];
                uint32_t o;
                if (TWO) o = (e & 1) ? two_level_half_fast<4>(src, tab[t]) : two_level_half_fast<0>(src, tab[t]);
                else o = (e & 1) ? sm_half_to_e4m3_fast<4>(src) : sm_half_to_e4m3_fast<0>(src);
                keep_here(o);
                eop[t][e] = o;
                if (e == 3) publish(buf ^ 1, t, 0, eop[t][0], eop[t][1], eop[t][2], eop[t][3]);
                if (e == 7) publish(buf ^ 1, t, 1, eop[t][4], eop[t][5], eop[t][6], eop[t][7]);
            }
            constexpr int ALU = ((SUM_IN_MFMA || st < 2) ? 0 : 4) + (EXPAND ? 4 : 0);
            if (j == 0 && f + 1 < WM) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // LDS reads of the next block
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                            // this step's MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, ALU, 0);                          // ALU work independent of it
            if (EXPAND && (e == 3 || e == 7)) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   // the publishing LDS write
            __builtin_amdgcn_sched_barrier(0);
        });
        if (!SUM_IN_MFMA) {
            fold(std::integral_constant<int, (STEPS - 2) / WN>{}, std::integral_constant<int, (STEPS - 2) % WN>{}, p_prev2);
            fold(std::integral_constant<int, WM - 1>{}, std::integral_constant<int, WN - 1>{}, p_prev);
        }
        __builtin_amdgcn_s_setprio(0);
        if (TWO) {
            // a band whose group holds a -8 (marked by the packer, rare): its operand again, this time with the pattern
            // 1000 put right -- after the steps, so that their instruction sequence stays one block
#pragma unroll
            for (int t = 0; t < EPW; ++t) {
                if (any_marked(cur.es[t])) {
                    const v8i o = slot_to_operand_two_level<true>(make_uint4(cur.raw[t][0], cur.raw[t][1], cur.raw[t][2], cur.raw[t][3]), tab[t]);
                    publish(buf ^ 1, t, 0, (uint32_t)o[0], (uint32_t)o[1], (uint32_t)o[2], (uint32_t)o[3]);
                    publish(buf ^ 1, t, 1, (uint32_t)o[4], (uint32_t)o[5], (uint32_t)o[6], (uint32_t)o[7]);
                }
            }
        }
        lds_dma_wait_all();                                      // this wavefront's copies and loads have landed ...
        __syncthreads();                                         // ... and so have everyone's; the stages just read are free
    };

    // A tile's start, first half: the copies of chunk 0's activations into stage 0, and the loads of chunk 0's nibbles
    // and scales and of chunk 1's nibbles (the copies first: the loads are then the younger operations, and the waits
    // the compiler puts in front of their first uses leave the copies alone).
    Set sa, sb;
    u32x4 raw0[EPW];
    float es0[EPW];                                              // two-level mode: scales of chunk 0's bands
    auto start_issue = [&]() {
#pragma unroll
        for (int q = 0; q < DPW; ++q) stage_page(c_begin, 0, q);
#pragma unroll
        for (int t = 0; t < EPW; ++t)
            raw0[t] = *reinterpret_cast<const W4A8_GLOBAL u32x4*>(uniform(ebase[t] + (int64_t)c_begin * 1024) + woff);
        if (TWO) {
#pragma unroll
            for (int t = 0; t < EPW; ++t) es0[t] = *reinterpret_cast<const W4A8_GLOBAL float*>(uniform(esbase[t] + (int64_t)(c_begin / cpg) * 64) + soff);
        }
        load_scales(sa, c_begin);
#pragma unroll
        for (int t = 0; t < EPW; ++t) {
            sa.raw[t] = u32x4{0u, 0u, 0u, 0u};
            sa.es[t] = 0.0f;
        }
        if (c_begin + 1 < c_end) load_raw(sa, c_begin + 1);
    };
    // second half: chunk 0's weight operands, expanded from registers, into stage 0; then everything has landed
    auto start_finish = [&]() {
#pragma unroll
        for (int t = 0; t < EPW; ++t) {
            const uint4 r = make_uint4(raw0[t][0], raw0[t][1], raw0[t][2], raw0[t][3]);
            const v8i o = TWO ? slot_to_operand_two_level<true>(r, two_level_table(es0[t])) : slot_to_operand<false>(r);
            publish(0, t, 0, (uint32_t)o[0], (uint32_t)o[1], (uint32_t)o[2], (uint32_t)o[3]);
            publish(0, t, 1, (uint32_t)o[4], (uint32_t)o[5], (uint32_t)o[6], (uint32_t)o[7]);
        }
        lds_dma_wait_all();
    };

    const float sx = ksplit > 1 ? 1.0f : *s_x;                   // partial sums are stored unscaled
    const float yq = (sizeof(OutT) == 1) ? *y_scale : 1.0f;      // FP8 output: the next layer's activation scale

    // Epilogue of the tile (em0, ebn), 16-token blocks f0 .. f1-1 of every wavefront row.
    auto epilogue = [&](int em0, int ebn, int esplit, auto F0, auto F1) {
        constexpr int f0 = decltype(F0)::value, f1 = decltype(F1)::value;
        const int n_block = ebn * BN;
        OutT* const yo = y + (int64_t)esplit * split_stride;     // this unit's share of the workspace (esplit = 0 without a split)
        if constexpr (DIRECT) {
            // Result lane: channel i of band j, tokens 4 kq .. 4 kq + 3 of block f.  Every wavefront turns its 16 tokens x
            // 16 WN channels of a block into row-major order in an LDS slab of its own (a wavefront's LDS accesses run in
            // order: no barrier, no wait beyond the one for the data) and stores 16 bytes per lane, whole row segments.
            constexpr int EB = (int)sizeof(OutT);
            constexpr int ROW_B = 16 * WN * EB, RSB = ROW_B + 16;    // bytes of a slab row, and its stride
            constexpr int SEGS = ROW_B / 16, ROWS_PER_STORE = 64 / SEGS, STORES = 16 / ROWS_PER_STORE;
            static_assert(WAVES * 16 * RSB <= (B_STAGES == 2 ? STAGE : A_STAGE), "the wavefronts' slabs fit stage 1");
            uint8_t* const slab = lds + STAGE + wave * (16 * RSB);
            const bool vec_ok = (ldy * EB) % 16 == 0 && reinterpret_cast<uintptr_t>(yo) % 16 == 0;
            const int n_wave = n_block + wn * WN * 16;               // first channel of the wavefront's bands
            const int seg = lane % SEGS, srow = lane / SEGS;
            float so[WN];                                            // output scale of the lane's channel of band j
#pragma unroll
            for (int j = 0; j < WN; ++j)
                so[j] = TWO ? sx * w_out[per_channel ? min(n_wave + j * 16 + i, N - 1) : 0] : sx;
#pragma unroll
            for (int f = f0; f < f1; ++f) {
#pragma unroll
                for (int j = 0; j < WN; ++j) {
                    if constexpr (EB == 2) {
                        // even lanes keep tokens 0, 1 and take the odd neighbour's, odd lanes keep tokens 2, 3: a lane then
                        // holds channels {i & ~1, i | 1} of two tokens, converted to bf16 by the hardware (round to nearest even)
                        typedef float f2 __attribute__((ext_vector_type(2)));
                        typedef __bf16 b2 __attribute__((ext_vector_type(2)));
                        const bool odd = (i & 1) != 0;
                        const uint32_t sel_lo = odd ? 0x05040100u : 0x01000504u, sel_hi = odd ? 0x07060302u : 0x03020706u;
                        const f2 t01 = {so[j] * acc[f][j][0], so[j] * acc[f][j][1]}, t23 = {so[j] * acc[f][j][2], so[j] * acc[f][j][3]};
                        const b2 c01 = __builtin_convertvector(t01, b2), c23 = __builtin_convertvector(t23, b2);
                        const uint32_t a = *reinterpret_cast<const uint32_t*>(&c01), b = *reinterpret_cast<const uint32_t*>(&c23);
                        const uint32_t own = odd ? b : a, nb = from_pair_lane(odd ? a : b);
                        uint8_t* p = slab + (4 * kq + (odd ? 2 : 0)) * RSB + (j * 16 + (i & ~1)) * 2;
                        *reinterpret_cast<uint32_t*>(p) = __builtin_amdgcn_perm(own, nb, sel_lo);
                        *reinterpret_cast<uint32_t*>(p + RSB) = __builtin_amdgcn_perm(own, nb, sel_hi);
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            *reinterpret_cast<float*>(slab + (4 * kq + r) * RSB + (j * 16 + i) * 4) = so[j] * acc[f][j][r];
                    }
                }
#pragma unroll
                for (int h = 0; h < STORES; ++h) {
                    const int row = h * ROWS_PER_STORE + srow;
                    const uint4 w = *reinterpret_cast<const uint4*>(slab + row * RSB + seg * 16);
                    const int m = em0 + (wm * WM + f) * 16 + row, n = n_wave + seg * (16 / EB);
                    if (m < M && n < N) {
                        OutT* dst = yo + (int64_t)m * ldy + n;
                        if (vec_ok && n + 16 / EB <= N) {
                            *reinterpret_cast<uint4*>(dst) = w;
                        } else {
                            const uint32_t e4[4] = {w.x, w.y, w.z, w.w};
                            for (int e = 0; e < 16 / EB && n + e < N; ++e) {
                                if constexpr (EB == 2) dst[e] = (uint16_t)(e4[e / 2] >> (16 * (e % 2)));
                                else dst[e] = __uint_as_float(e4[e]);
                            }
                        }
                    }
                }
            }
        } else {
            static_assert(!TWO || DIRECT, "the two-level mode has float32 and bf16 outputs only");
            // E4M3 outputs: per round the workgroup turns block f of every wavefront row into row-major order in LDS
            // (stage 1, which nothing else uses between two tiles) and stores whole row segments
            SlabT* slab = reinterpret_cast<SlabT*>(lds + STAGE);
            constexpr int VEC = SILU ? 16 : 16 / sizeof(SlabT);  // outputs per 16-byte store
            constexpr int UPR = (SILU ? BN / 2 : BN) / VEC;      // 16-byte units per row
            const bool vec_ok = (ldy % VEC == 0) && (reinterpret_cast<uintptr_t>(y) % 16 == 0);
#pragma unroll
            for (int f = f0; f < f1; ++f) {
#pragma unroll
                for (int j = 0; j < WN; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        slab[(wm * 16 + 4 * kq + r) * RS + (wn * WN + j) * 16 + i] = OutCast<SlabT>::cast(sx * acc[f][j][r], yq);
                __syncthreads();
                for (int u = tid; u < SLAB_ROWS * UPR; u += THREADS) {
                    const int row = u / UPR, col = (u % UPR) * VEC;
                    const int m = em0 + ((row >> 4) * WM + f) * 16 + (row & 15);
                    if constexpr (SILU) {
                        // 16 outputs of one band pair: gate = slab columns 32p .. 32p+15, up = 32p+16 .. 32p+31 (p = col / 16)
                        const int n_out = n_block / 2 + col;
                        if (m < M && n_out < N / 2) {
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
                        if (m < M && n < N) {
                            OutT* dst = y + (int64_t)m * ldy + n;
                            const OutT* src = reinterpret_cast<const OutT*>(slab) + row * RS + col;
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
    };

    set_tile(v);
    start_issue();
    start_finish();
    __syncthreads();
    for (;;) {
#pragma unroll
        for (int f = 0; f < WM; ++f)
#pragma unroll
            for (int j = 0; j < WN; ++j) acc[f][j] = v4f{0.f, 0.f, 0.f, 0.f};
        for (int c = c_begin; c < c_end; c += 2) {
            chunk(c, sa, sb);
            if (c + 1 < c_end) chunk(c + 1, sb, sa);
        }
        // The loop's last barrier has passed: both stages are free.  The next tile's first copies and loads go out
        // before this tile's epilogue and are waited for in its middle; they touch stage 0 only (the slab epilogue
        // works in stage 1).
        const int em0 = m0, ebn = bn;
        const int esplit = split;
        const int v_next = v + nx;
        const bool more = v_next < v_end;
        if (more) {
            set_tile(v_next);
            start_issue();
        }
        epilogue(em0, ebn, esplit, std::integral_constant<int, 0>{}, std::integral_constant<int, WM / 2>{});
        if (more) start_finish();
        epilogue(em0, ebn, esplit, std::integral_constant<int, WM / 2>{}, std::integral_constant<int, WM>{});
        if (!more) break;
        __syncthreads();
        v = v_next;
    }
}

// Sum of the K ranges' partial sums in the order of the ranges (fixed, so the result does not depend on which workgroup
// finished first), then the output scale and cast of the layer: y[m, n] = cast(s_x * sum_s partial[s][m][n]).
template <typename OutT>
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const float* __restrict__ partial, int ksplit, int64_t split_stride,
                                                            int64_t ldw, int M, int N, const float* __restrict__ s_x,
                                                            OutT* __restrict__ y, int64_t ldy, const float* __restrict__ y_scale) {
    const int n4 = (N + 3) / 4;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)M * n4) return;
    const int m = (int)(idx / n4), n = (int)(idx % n4) * 4;
    const float sx = *s_x;
    const float yq = (sizeof(OutT) == 1) ? *y_scale : 1.0f;
    const float* p = partial + (int64_t)m * ldw + n;             // ldw is a multiple of 4: a float4 stays inside the row
    float4 sum = *reinterpret_cast<const float4*>(p);
    for (int s = 1; s < ksplit; ++s) {
        const float4 t = *reinterpret_cast<const float4*>(p + (int64_t)s * split_stride);
        sum.x += t.x; sum.y += t.y; sum.z += t.z; sum.w += t.w;
    }
    const float v[4] = {sum.x, sum.y, sum.z, sum.w};
    for (int e = 0; e < 4 && n + e < N; ++e) y[(int64_t)m * ldy + n + e] = OutCast<OutT>::cast(sx * v[e], yq);
}

struct SplitArgs {
    int ksplit = 1, cps = 0;
    int64_t split_stride = 0;
};

template <typename OutT, int WGM, int WGN, int WM, int WN>
void launch_cfg(const LinearArgs& a, dim3 grid, int grid_m, int grid_n, int group_m, const SplitArgs& sp, hipStream_t st) {
#define W4A8_MFMA2D(MODEV)                                                                                                     \
    hipLaunchKernelGGL((linear_mfma2d_kernel<OutT, WGM, WGN, WM, WN, MODEV>), grid, dim3(64 * WGM * WGN), 0, st, a.x8, a.M, a.ldx8, \
                       a.s_x, a.packed, a.scales, a.N, a.n_tiles, a.C, a.cpg, a.NG, static_cast<OutT*>(a.y), a.ldy, grid_m,       \
                       grid_n, group_m, a.y_scale, sp.ksplit, sp.cps > 0 ? sp.cps : a.C, sp.split_stride, a.w_out, a.per_channel)
    if constexpr (sizeof(OutT) == 1) {                           // FP8 output exists for the code-exact mode only
        W4A8_MFMA2D(MODE_CODE_EXACT);
    } else {
        if (a.mode == MODE_POW2) W4A8_MFMA2D(MODE_POW2);
        else if (a.mode == MODE_TWO_LEVEL) W4A8_MFMA2D(MODE_TWO_LEVEL);
        else W4A8_MFMA2D(MODE_CODE_EXACT);
    }
#undef W4A8_MFMA2D
}

template <int WGM, int WGN, int WM, int WN>
void launch_out(const LinearArgs& a, int ydt, dim3 grid, int grid_m, int grid_n, int group_m, const SplitArgs& sp, hipStream_t st) {
    if (ydt == W4A8_F32) launch_cfg<float, WGM, WGN, WM, WN>(a, grid, grid_m, grid_n, group_m, sp, st);
    else if (ydt == YDT_SILU_E4M3) launch_cfg<SiluFp8, WGM, WGN, WM, WN>(a, grid, grid_m, grid_n, group_m, sp, st);
    else if (ydt == YDT_E4M3) launch_cfg<uint8_t, WGM, WGN, WM, WN>(a, grid, grid_m, grid_n, group_m, sp, st);
    else launch_cfg<uint16_t, WGM, WGN, WM, WN>(a, grid, grid_m, grid_n, group_m, sp, st);
}

}  // namespace

// Built workgroup tiles {tokens, channels}: cfg 0 = 512 x 128, 1 = 256 x 256, 2 = 256 x 128, 3 = 128 x 256, 5 = 128 x 128
// (eight wavefronts, one workgroup per compute unit); 4 = 256 x 128 with four wavefronts, two workgroups per compute unit.
bool mfma2d_tile(int cfg, int& bm, int& bn) {
    static const int t[6][2] = {{512, 128}, {256, 256}, {256, 128}, {128, 256}, {256, 128}, {128, 128}};
    if (cfg < 0 || cfg > 5) return false;
    bm = t[cfg][0];
    bn = t[cfg][1];
    return true;
}

// cfg: a tile of mfma2d_tile; group_m = token blocks per super-column of the block order (0: chosen); workgroups = size
// of the persistent grid (0: one per compute unit); ksplit > 1: K is multiplied in that many ranges by different workgroups
// whose float32 partial sums go through `workspace` (mfma2d_splitk_bytes) and are summed by a second launch.
int launch_linear_mfma2d(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x, const uint8_t* packed,
                         const float* scales, int64_t N, int32_t G, void* y, w4a8_dtype ydt, int64_t ldy, int cfg,
                         int group_m, int workgroups, int mode, const float* y_scale, hipStream_t st, int ksplit,
                         void* workspace, const float* w_out, int per_channel) {
    if (mode != MODE_CODE_EXACT && mode != MODE_POW2 && mode != MODE_TWO_LEVEL) return W4A8_ERR_DTYPE;
    if (mode == MODE_TWO_LEVEL && (!w_out || ksplit > 1 || ((int)ydt != W4A8_F32 && (int)ydt != W4A8_BF16))) return W4A8_ERR_DTYPE;
    if (((int)ydt == YDT_E4M3 || (int)ydt == YDT_SILU_E4M3) && (mode != MODE_CODE_EXACT || !y_scale)) return W4A8_ERR_DTYPE;
    if ((int)ydt == YDT_SILU_E4M3 && N % 32 != 0) return W4A8_ERR_SHAPE;
    int bm, bn;
    if (!mfma2d_tile(cfg, bm, bn)) return W4A8_ERR_SHAPE;
    const int C = (int)(K / 128), cpg = G / 128, NG = (int)(K / G);
    const int n_tiles = (int)((N + 15) / 16);
    const int grid_m = (int)((M + bm - 1) / bm), grid_n = (int)((N + bn - 1) / bn);
    if (ksplit < 1) ksplit = 1;
    if (ksplit > 1 && (ksplit > C || !workspace || (int)ydt == YDT_SILU_E4M3)) return W4A8_ERR_SHAPE;
    SplitArgs sp;
    if (ksplit > 1) {
        sp.cps = (C + ksplit - 1) / ksplit;
        ksplit = (C + sp.cps - 1) / sp.cps;                     // no empty range
        sp.ksplit = ksplit;
        sp.split_stride = M * mfma2d_splitk_ldw(N);
    }
    const int64_t total = (int64_t)grid_m * grid_n * ksplit;
    if (total > (1 << 30)) return W4A8_ERR_SHAPE;
    if (ldx8 >= (1 << 23) || ldy >= (1 << 20) || N >= (1 << 20)) return W4A8_ERR_SHAPE;   // 32-bit byte offsets inside a tile
    if (group_m <= 0) {
        // One XCD runs 32 workgroups at a time; per chunk they pull rows * 128 bytes of activations and columns * 64
        // bytes of nibbles through its L2, least for a rectangle with about twice as many columns as rows:
        // rows^2 * 2 = 32 * bm * bn
        group_m = (int)(sqrtf(16.0f * (float)bm * (float)bn) / (float)bm + 0.5f);
        if (group_m < 1) group_m = 1;
    }
    if (group_m > grid_m) group_m = grid_m;
    if (workgroups <= 0) workgroups = cfg == 4 ? 512 : 256;      // one per compute unit (160 KB of LDS each), or two
    workgroups = (workgroups + XCDS2 - 1) / XCDS2 * XCDS2;
    const int64_t needed = (total + XCDS2 - 1) / XCDS2 * XCDS2;
    if (workgroups > needed) workgroups = (int)needed;
    const dim3 grid((unsigned)workgroups);
    LinearArgs a{x8, (int)M, ldx8, s_x, packed, scales, (int)N, n_tiles, C, cpg, NG, y, ldy, w_out, per_channel, mode, y_scale};
    int kernel_ydt = (int)ydt;
    if (ksplit > 1) {                                            // the tiles go to the workspace as unscaled float32
        a.y = workspace;
        a.ldy = mfma2d_splitk_ldw(N);
        kernel_ydt = W4A8_F32;
    }
    switch (cfg) {
        case 0: launch_out<4, 2, 8, 4>(a, kernel_ydt, grid, grid_m, grid_n, group_m, sp, st); break;
        case 1: launch_out<2, 4, 8, 4>(a, kernel_ydt, grid, grid_m, grid_n, group_m, sp, st); break;
        case 2: launch_out<4, 2, 4, 4>(a, kernel_ydt, grid, grid_m, grid_n, group_m, sp, st); break;
        case 3: launch_out<2, 4, 4, 4>(a, kernel_ydt, grid, grid_m, grid_n, group_m, sp, st); break;
        case 4: launch_out<2, 2, 8, 4>(a, kernel_ydt, grid, grid_m, grid_n, group_m, sp, st); break;
        default: launch_out<2, 4, 4, 2>(a, kernel_ydt, grid, grid_m, grid_n, group_m, sp, st); break;
    }
    if (int e = launch_status()) return e;
    if (ksplit > 1) {
        const int64_t work = M * ((N + 3) / 4);
        const dim3 rgrid((unsigned)((work + 255) / 256));
        const float* ws = static_cast<const float*>(workspace);
#define W4A8_REDUCE(T)                                                                                                       \
    hipLaunchKernelGGL((splitk_reduce_kernel<T>), rgrid, dim3(256), 0, st, ws, ksplit, sp.split_stride, mfma2d_splitk_ldw(N), (int)M, \
                       (int)N, s_x, static_cast<T*>(y), ldy, y_scale)
        if (ydt == W4A8_F32) W4A8_REDUCE(float);
        else if ((int)ydt == YDT_E4M3) W4A8_REDUCE(uint8_t);
        else W4A8_REDUCE(uint16_t);
#undef W4A8_REDUCE
        return launch_status();
    }
    return W4A8_OK;
}

}  // namespace w4a8
