// W4A8 linear layer for few tokens (M <= 64): the memory-bound regime of Sec. 1, where the time is the time to
// stream the 4-bit weights from HBM once.
//
// Work split: a workgroup owns NT tiles of 16 output channels; its wavefronts split K between them (each takes a
// contiguous run of 128-deep chunks, which is contiguous memory in the tiled format) and their partial results
// are summed through LDS.  Per chunk a wavefront issues one 16-byte load per lane and tile (the 1 KiB tile is read
// fully coalesced), expands the sign-magnitude nibbles to E4M3 in registers (Eq. 10; four ALU ops per four weights,
// plus a fix-up for -8 on chunks whose scales the packer has marked) and feeds them as the column operand of one
// 16x16x128 FP8 MFMA per (tile, 16-token block); the activations are the row operand, loaded straight from global
// memory (they are small and stay in cache).  A result lane therefore holds ONE channel (and four tokens): the
// chunk's partial product is scaled in fp32 by a group scale that is a single 4-byte load per lane -- the vector
// memory path returns 64 bytes per clock to a compute unit whatever the addresses, so a float4 of scales per lane
// (what the other operand order needs) costs it as much as the kilobyte of nibbles does.
// Several chunks' loads are in flight ahead of the current chunk's arithmetic.
#include "w4a8_device.hpp"
#include "w4a8_internal.hpp"

namespace w4a8 {
namespace {

constexpr int RED_STRIDE = 65;      // floats per (wave, register) row in LDS: 64 lanes + 1 to spread banks

template <int MT, int NT>
struct ChunkLoads {
    uint4 w[NT];          // packed nibbles: this lane's slot of each tile
    float s[NT];          // group scale of the lane's channel (the one whose nibbles it expands and whose results it holds)
    uint4 x[MT][2];       // 32 activation bytes per 16-token block
    uint32_t z[NT];       // asymmetric format: the zero-point of the lane's channel
};

// larger register tiles run with fewer wavefronts per workgroup (the launcher enforces it), which raises the
// register budget per lane: 128 at 1024 threads, 256 at 512 and below; the asymmetric format's zero-point terms need
// the larger budget from two tiles on
// (the fused gate|up form at 17..32 tokens -- two token blocks x two bands, code-exact mode -- fits the smaller budget
// as well, 119 registers, and takes it, so that it can split K over as many wavefronts as the plain layer does)
constexpr int max_threads(int tiles, bool asym = false, bool fused_gate_up_2x2 = false) {
    return (tiles <= (asym ? 1 : 2) || fused_gate_up_2x2) ? 1024 : (tiles <= 8 ? 512 : 256);
}

// DEPTH = chunks in flight per wavefront (a ring of register buffers).  MODE_CODE_EXACT: signed codes, group scales
// applied to the partial sums in fp32.  MODE_TWO_LEVEL: the weight operand is nearest_E4M3(code * s8[n,g]), the sum over
// the wavefront's share of K stays in the MFMA accumulator and the output is scaled by s_x * w_out[n] (w_out[0] when
// per_channel is 0).  MODE_ASYM: unsigned codes with per-group zero-points, the weight operand is the integer
// code - zero_point, scales as in the code-exact mode; `scales` then points at the 80-byte records of scales and
// zero-points; MODE_ASYM_TWO: the same records with FP8-domain scales, the weight operand is
// nearest_E4M3((code - zero_point) * s8[n,g]), accumulation and output scale as in MODE_TWO_LEVEL.  MODE_POW2: signed codes, the group scale is a power of two that the matrix unit applies itself
// (block-scaled MFMA); the sum over the wavefront's share of K stays in the MFMA accumulator.
// XQ != 0 (few tokens, M * K <= 64 KiB): the activation quantization of Eq. 13 is folded in.  `x8` then is the float32
// (XQ = 1) or bf16 (XQ = 2) activation matrix itself, row stride ldx8 ELEMENTS; every workgroup quantizes all of it into
// LDS while its first weight loads are in flight (the same single float32 division and rounding per element as the
// stand-alone kernel), and the main loop takes its activation operands from there.  Workgroup 0 also writes the
// codes to x8_out (row stride K) when that is not null.
template <int MT, int NT, int DEPTH, typename OutT, int MODE, int XQ>
__global__ void __launch_bounds__(max_threads(MT * NT, MODE == MODE_ASYM || MODE == MODE_ASYM_TWO,
                                               OutKind<OutT>::SILU && MT == 2 && NT == 2)) linear_skinny_kernel(
    const uint8_t* __restrict__ x8, int M, int64_t ldx8, const float* __restrict__ s_x,
    const uint8_t* __restrict__ packed, const float* __restrict__ scales, int N, int n_tiles, int C, int cpg, int NG,
    OutT* __restrict__ y, int64_t ldy, int cpw, const float* __restrict__ w_out, int per_channel,
    const float* __restrict__ y_scale, uint8_t* __restrict__ x8_out) {
    constexpr bool ASYM2 = MODE == MODE_ASYM_TWO;                // asymmetric records, two-level bytes, sum kept in the MFMA
    constexpr bool TWO = MODE == MODE_TWO_LEVEL, ASYM = MODE == MODE_ASYM, POW2 = MODE == MODE_POW2;
    constexpr bool OUT_SCALED = TWO || ASYM2;                    // output scaled by s_x * w_out[n]
    constexpr int REC = (ASYM || ASYM2) ? ASYM_RECORD_BYTES : 64;   // bytes of scales (and zero-points) per tile and group
    extern __shared__ float red[];
    // the output scales are only needed at the very end; asked for here, their (possibly cold) loads are long back by then
    const float sx = *s_x;
    const float yq = (sizeof(OutT) == 1) ? *y_scale : 1.0f;      // FP8 output: the next layer's activation scale
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);     // wave-uniform: keeps the loop scalar
    const int waves = blockDim.x >> 6;
    const int i = lane & 15, kq = lane >> 4;
    const int t0 = blockIdx.x * NT;
    const int c_begin = wave * cpw;
    const int c_end = min(C, c_begin + cpw);

    // wave-uniform base pointers (advance by one chunk per step) plus small per-lane offsets
    const uint8_t* wbase[NT];
    const uint8_t* sbase[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int t = min(t0 + j, n_tiles - 1);                  // tiles past the end reload the last one; not stored
        wbase[j] = packed + ((int64_t)t * C + c_begin) * 1024;
        sbase[j] = reinterpret_cast<const uint8_t*>(scales) + (int64_t)t * NG * REC;
    }
    const uint32_t woff = lane * 16, soff = i * 4;
    const uint8_t* xp[MT];                                       // XQ == 0: the lane's activation bytes in global memory
    uint32_t xo[MT];                                             // XQ != 0: their offset in the LDS copy, [M][K] bytes
    uint8_t* xl = reinterpret_cast<uint8_t*>(red);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = min(mt * 16 + i, M - 1);                   // rows past the end reload the last one; not stored
        xp[mt] = x8 + (int64_t)m * ldx8 + kq * 32 + (int64_t)c_begin * 128;
        xo[mt] = (uint32_t)m * (uint32_t)(C * 128) + kq * 32 + c_begin * 128;
    }
    int g = c_begin / cpg, g_left = cpg - (c_begin - g * cpg);   // current group and chunks left in it

    auto load_x = [&](ChunkLoads<MT, NT>& L) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (XQ) {
                L.x[mt][0] = *reinterpret_cast<const uint4*>(xl + xo[mt]);
                L.x[mt][1] = *reinterpret_cast<const uint4*>(xl + xo[mt] + 16);
                xo[mt] += 128;
            } else {
                L.x[mt][0] = *reinterpret_cast<const uint4*>(xp[mt]);
                L.x[mt][1] = *reinterpret_cast<const uint4*>(xp[mt] + 16);
                xp[mt] += 128;
            }
        }
    };
    auto load_ws = [&](ChunkLoads<MT, NT>& L) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            L.w[j] = *reinterpret_cast<const uint4*>(wbase[j] + woff);
            L.s[j] = *reinterpret_cast<const float*>(sbase[j] + (int64_t)g * REC + soff);
            L.z[j] = (ASYM || ASYM2) ? (uint32_t)sbase[j][(int64_t)g * REC + 64 + i] : 0u;
            wbase[j] += 1024;
        }
        if (--g_left == 0) { ++g; g_left = cpg; }
    };
    auto load_chunk = [&](ChunkLoads<MT, NT>& L) {
        load_ws(L);
        load_x(L);
    };

    v4f acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[mt][j] = v4f{0.f, 0.f, 0.f, 0.f};

    auto compute_chunk = [&](const ChunkLoads<MT, NT>& L) {
        v8i xop[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const uint4 a = L.x[mt][0], b = L.x[mt][1];
            xop[mt] = v8i{(int)a.x, (int)a.y, (int)a.z, (int)a.w, (int)b.x, (int)b.y, (int)b.z, (int)b.w};
        }
        // asymmetric format: sum_k x over the chunk, per token, from an MFMA against an operand of ones (every column
        // of the result is that sum: the lane gets the sums of its own four tokens)
        v4f xs[MT];
        if (ASYM) {
            const v8i ones = v8i{0x38383838, 0x38383838, 0x38383838, 0x38383838, 0x38383838, 0x38383838, 0x38383838, 0x38383838};
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xs[mt] = mfma_16x16x128_e4m3(xop[mt], ones, v4f{0.f, 0.f, 0.f, 0.f});
        }
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const float s = L.s[j];
            // a marked scale (sign bit) on any of the band's 16 channels: this chunk's tile may hold -8
            const bool m8 = !ASYM && !ASYM2 && any_marked(s);
            v8i wop;
            if (TWO) {
                const MagTable tab = two_level_table(s);
                wop = m8 ? slot_to_operand_two_level<true>(L.w[j], tab) : slot_to_operand_two_level<false>(L.w[j], tab);
            } else if (ASYM2) {
                wop = slot_to_operand_asym(L.w[j], asym_two_level_table(L.z[j], s));
            } else if (ASYM) {
                wop = slot_to_operand_half_offset(L.w[j]);       // code - 7.5
            } else {
                wop = slot_to_operand<false>(L.w[j]);
                if (m8) {                                        // wave-uniform, rare
#pragma unroll
                    for (int e = 0; e < 8; ++e) wop[e] = (int)sm_fix_minus_eight((uint32_t)wop[e]);
                }
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if (TWO || ASYM2) {
                    acc[mt][j] = mfma_16x16x128_e4m3(xop[mt], wop, acc[mt][j]);
                    continue;
                }
                if (POW2) {
                    acc[mt][j] = mfma_16x16x128_e4m3_scaled(xop[mt], wop, acc[mt][j], E8M0_ONE, e8m0_of(s));
                    continue;
                }
                v4f p = mfma_16x16x128_e4m3(xop[mt], wop, v4f{0.f, 0.f, 0.f, 0.f});
                if (ASYM) {                                      // sum x (u - z) = sum x (u - 7.5) + (7.5 - z) sum x
                    const float zf = 7.5f - (float)L.z[j];
                    p[0] = fmaf(zf, xs[mt][0], p[0]);
                    p[1] = fmaf(zf, xs[mt][1], p[1]);
                    p[2] = fmaf(zf, xs[mt][2], p[2]);
                    p[3] = fmaf(zf, xs[mt][3], p[3]);
                }
                const float sa = fabsf(s);                       // the sign bit is the packer's mark, not part of the scale
                acc[mt][j][0] = fmaf(sa, p[0], acc[mt][j][0]);
                acc[mt][j][1] = fmaf(sa, p[1], acc[mt][j][1]);
                acc[mt][j][2] = fmaf(sa, p[2], acc[mt][j][2]);
                acc[mt][j][3] = fmaf(sa, p[3], acc[mt][j][3]);
            }
        }
    };

    // DEPTH chunks in flight per wavefront: a ring of register buffers, refilled in chunk order right after use.
    // The steady-state loop refills unconditionally: with a load that may or may not have been issued the compiler has
    // to wait for the youngest load before every chunk (vmcnt(0)), which exposes the memory latency again; the last
    // chunks, whose refills fall off the end of the wavefront's K range, run in a separate tail.
    {
        ChunkLoads<MT, NT> ring[DEPTH];
        if (XQ) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d)
                if (c_begin + d < c_end) load_ws(ring[d]);       // the first weights are on their way ...
            // ... while the workgroup quantizes the activations (Eq. 13), 16 elements per thread and turn
            const int k16 = C * 8;                               // 16-element units per row
            for (int u = threadIdx.x; u < M * k16; u += blockDim.x) {
                const int m = u / k16, k = (u - m * k16) * 16;
                float v[16];
                if (XQ == 1) Load16<float>::load(reinterpret_cast<const float*>(x8) + (int64_t)m * ldx8 + k, v);
                else Load16<uint16_t>::load(reinterpret_cast<const uint16_t*>(x8) + (int64_t)m * ldx8 + k, v);
                uint4 o;
                o.x = quant4(v[0], v[1], v[2], v[3], sx);
                o.y = quant4(v[4], v[5], v[6], v[7], sx);
                o.z = quant4(v[8], v[9], v[10], v[11], sx);
                o.w = quant4(v[12], v[13], v[14], v[15], sx);
                *reinterpret_cast<uint4*>(xl + (uint32_t)m * (uint32_t)(C * 128) + k) = o;
                if (x8_out != nullptr && blockIdx.x == 0) *reinterpret_cast<uint4*>(x8_out + (int64_t)m * (C * 128) + k) = o;
            }
            __syncthreads();
#pragma unroll
            for (int d = 0; d < DEPTH; ++d)
                if (c_begin + d < c_end) load_x(ring[d]);
        } else {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d)
                if (c_begin + d < c_end) load_chunk(ring[d]);
        }
        int c = c_begin;
        for (; c + 2 * DEPTH <= c_end; c += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                compute_chunk(ring[d]);
                load_chunk(ring[d]);
            }
        }
        for (; c < c_end; c += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                if (c + d < c_end) {
                    compute_chunk(ring[d]);
                    if (c + d + DEPTH < c_end) load_chunk(ring[d]);
                }
            }
        }
    }

    if (XQ) __syncthreads();                                     // the partial sums below reuse the activations' LDS
    // sum the wavefronts' partials through LDS: red[wave][e = (mt*NT + j)*4 + r][lane]
    constexpr int E = MT * NT * 4;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[(wave * E + (mt * NT + j) * 4 + r) * RED_STRIDE + lane] = acc[mt][j][r];
    __syncthreads();

    constexpr int COLS = 16 * NT;                                // output channels of this workgroup
    if constexpr (OutKind<OutT>::SILU) {
        // gate|up with SiLU*mul and the next quantization folded in: tiles 2p and 2p+1 of the workgroup are the gate and
        // up rows of the same 16 channels; one thread per output byte
        constexpr int HALF = COLS / 2;
        uint8_t* h8 = reinterpret_cast<uint8_t*>(y);
        for (int idx = threadIdx.x; idx < MT * 16 * HALF; idx += blockDim.x) {
            const int col = idx % HALF, row = idx / HALF;
            const int p = col >> 4, nl = col & 15, mt = row >> 4, ml = row & 15;
            const int src_lane = nl + 16 * (ml >> 2);            // lane = channel + 16 * (token / 4), register = token % 4
            const int eg = (mt * NT + 2 * p) * 4 + (ml & 3), eu = (mt * NT + 2 * p + 1) * 4 + (ml & 3);
            float sg = 0.0f, su = 0.0f;
            for (int w = 0; w < waves; ++w) {
                sg += red[(w * E + eg) * RED_STRIDE + src_lane];
                su += red[(w * E + eu) * RED_STRIDE + src_lane];
            }
            const int m = mt * 16 + ml, n_out = (t0 / 2) * 16 + col;
            if (m < M && n_out < N / 2) {
                const float g = bf16_bits_to_f32(f32_to_bf16_bits(sx * sg)), u = bf16_bits_to_f32(f32_to_bf16_bits(sx * su));
                h8[(int64_t)m * ldy + n_out] = quantize_one(bf16_bits_to_f32(f32_to_bf16_bits(silu_mul_f32(g, u))), yq);
            }
        }
    } else {
        for (int idx = threadIdx.x; idx < MT * 16 * COLS; idx += blockDim.x) {
            const int col = idx % COLS, row = idx / COLS;            // channel fastest: consecutive threads, consecutive y
            const int j = col >> 4, nl = col & 15, mt = row >> 4, ml = row & 15;
            const int e = (mt * NT + j) * 4 + (ml & 3), src_lane = nl + 16 * (ml >> 2);   // lane = channel + 16 * (token / 4)
            float sum = 0.0f;
            for (int w = 0; w < waves; ++w) sum += red[(w * E + e) * RED_STRIDE + src_lane];
            const int m = mt * 16 + ml, n = (t0 + j) * 16 + nl;
            if (m < M && n < N) y[(int64_t)m * ldy + n] = OutCast<OutT>::cast((OUT_SCALED ? sx * w_out[per_channel ? n : 0] : sx) * sum, yq);
        }
    }
}

template <int MT, int NT, typename OutT>
int launch_one(const LinearArgs& a, int depth, int waves, hipStream_t st) {
    const int grid = (a.n_tiles + NT - 1) / NT;
    const int cpw = (a.C + waves - 1) / waves;
    const size_t lds = (size_t)waves * MT * NT * 4 * RED_STRIDE * sizeof(float);
    constexpr int DEEP = (MT * NT == 1) ? 4 : 2;                 // deeper ring while the registers allow it
#define W4A8_SKINNY_X(DEPTHV, MODEV, XQV, LDSV)                                                                              \
    hipLaunchKernelGGL((linear_skinny_kernel<MT, NT, DEPTHV, OutT, MODEV, XQV>), dim3(grid), dim3(waves * 64), LDSV, st, a.x8,   \
                       a.M, a.ldx8, a.s_x, a.packed, a.scales, a.N, a.n_tiles, a.C, a.cpg, a.NG, static_cast<OutT*>(a.y), a.ldy, \
                       cpw, a.w_out, a.per_channel, a.y_scale, a.x8_out)
#define W4A8_SKINNY(DEPTHV, MODEV) W4A8_SKINNY_X(DEPTHV, MODEV, 0, lds)
    if (a.xq != 0) {                                             // activation quantization folded in: few tokens; float32, bf16 or FP8 outputs
        if constexpr (MT == 1 && NT <= 2 && !OutKind<OutT>::SILU) {
            if (a.mode != MODE_CODE_EXACT) return W4A8_ERR_SHAPE;
            const size_t xbytes = (size_t)a.M * a.C * 128;
            const size_t both = lds > xbytes ? lds : xbytes;
            if (a.xq == 1) W4A8_SKINNY_X(2, MODE_CODE_EXACT, 1, both);
            else W4A8_SKINNY_X(2, MODE_CODE_EXACT, 2, both);
            return launch_status();
        } else {
            return W4A8_ERR_SHAPE;
        }
    }
    if constexpr (sizeof(OutT) == 1) {                           // FP8 output exists for the code-exact mode only
        W4A8_SKINNY(2, MODE_CODE_EXACT);
        return launch_status();
    } else {
    if (a.mode == MODE_TWO_LEVEL)
        W4A8_SKINNY(2, MODE_TWO_LEVEL);
    else if (a.mode == MODE_ASYM)
        W4A8_SKINNY(2, MODE_ASYM);
    else if (a.mode == MODE_POW2)
        W4A8_SKINNY(2, MODE_POW2);
    else if (a.mode == MODE_ASYM_TWO)
        W4A8_SKINNY(2, MODE_ASYM_TWO);
    else if (depth == DEEP)
        W4A8_SKINNY(DEEP, MODE_CODE_EXACT);
    else
        W4A8_SKINNY(2, MODE_CODE_EXACT);
    return launch_status();
    }
#undef W4A8_SKINNY
#undef W4A8_SKINNY_X
}

template <int MT, typename OutT>
int launch_nt(const LinearArgs& a, int nt, int depth, int waves, hipStream_t st) {
    switch (nt) {
        case 1:
            if constexpr (OutKind<OutT>::SILU) return W4A8_ERR_SHAPE;   // gate and up tiles come in pairs
            else return launch_one<MT, 1, OutT>(a, depth, waves, st);
        case 2: return launch_one<MT, 2, OutT>(a, depth, waves, st);
        case 4: return launch_one<MT, 4, OutT>(a, depth, waves, st);
    }
    return W4A8_ERR_SHAPE;
}

template <typename OutT>
int launch_mt(const LinearArgs& a, int mt, int nt, int depth, int waves, hipStream_t st) {
    switch (mt) {
        case 1: return launch_nt<1, OutT>(a, nt, depth, waves, st);
        case 2: return launch_nt<2, OutT>(a, nt, depth, waves, st);
        default: return launch_nt<4, OutT>(a, nt, depth, waves, st);
    }
}

}  // namespace

// Launch shape of the skinny kernel for a layer, from sweeps over the Llama-3-8B/70B layer shapes with the weights coming
// from HBM (requested values other than 0 are kept):
//  - two bands per wavefront when the activation operand is wide enough to be worth sharing (M > 8 on layers
//    with enough bands) or when the layer is large enough that fewer, longer-running workgroups ramp better;
//  - four bands per wavefront from 17 tokens on when the layer is very wide (every chunk of activations a wavefront
//    loads is then 2 KB or more, against 1 KB of nibbles per band), with fewer, longer-running wavefronts;
//  - up to 16 tokens, a grid between one and two workgroups per compute unit (256 of them) leaves half of the chip with
//    twice the work of the other half: one more doubling of the bands per wavefront brings it to at most one each;
//  - split K over as many wavefronts (a power of two) as it takes to have ~16384 (~2400 for M > 8) of them in flight;
//  - up to 8 tokens on long rows (K >= 8192) with more workgroups than the chip holds at once: eight wavefronts, each
//    with four chunks in flight where that ring is built (a workgroup's wavefronts start one after the other, about
//    60 ns apart, so half as many of them have their loads under way sooner).
// The split of K (the number of wavefronts) never depends on the output type or on whether the activation quantization is
// folded in: the fused forms add up the same partial sums in the same order as the plain layer and give the same bytes.
// Returns false for a combination that is not built.
bool skinny_launch_shape(int64_t M, int64_t K, int64_t N, int ydt, int mode, int xq, int& nt, int& waves, int& depth) {
    const int C = (int)(K / 128);
    const int n_tiles = (int)((N + 15) / 16);
    const int mt = (M <= 16) ? 1 : (M <= 32) ? 2 : 4;
    const bool wide_many = M > 16 && n_tiles >= 1024;
    const bool auto_nt = nt == 0;
    bool long_rows = false;
    if (auto_nt) {
        nt = wide_many ? 4 : ((M > 8 && n_tiles >= 384) || (int64_t)n_tiles * C >= 100000) ? 2 : 1;
        const int grid = (n_tiles + nt - 1) / nt;
        if (mt == 1 && grid > 256 && grid < 512 && nt < 4) nt *= 2;
        long_rows = waves == 0 && nt == 1 && M <= 8 && C >= 64 && n_tiles >= 512 && mode == MODE_CODE_EXACT;
    }
    if (nt != 1 && nt != 2 && nt != 4) return false;
    if (long_rows) waves = 8;
    if (waves == 0) {
        const int grid = (n_tiles + nt - 1) / nt;
        // (the two-level and power-of-two formats measured faster with half as many at few tokens: gate|up of
        // Llama-3-8B at one token 4.4 against 4.0 TB/s and 4.7 against 4.4)
        const bool many = mode == MODE_CODE_EXACT || mode == MODE_ASYM;
        const int target = (wide_many && nt == 4) ? (M > 32 ? 896 : 2048) : M > 8 ? 2400 : many ? 16384 : 8192;
        const float want = (float)target / (float)grid;
        waves = 2;                                               // the power of two nearest to `want` (ratio-wise), 2..16:
        while (waves < 16 && (float)(waves * waves * 2) < want * want) waves *= 2;
        // ... and no wavefront streams more than 64 KB of nibbles (the largest layers want more of them in flight)
        while (waves < 16 && (int64_t)n_tiles * C * 1024 > (int64_t)grid * waves * 65536) waves *= 2;   // odd counts split K unevenly and measured slower
    }
    if (waves > C) waves = C;
    const bool asym = mode == MODE_ASYM || mode == MODE_ASYM_TWO;
    // LDS and registers of the plain layer bound its wavefronts; every other form takes that count, or fewer where its
    // own kernel holds fewer
    const int plain_cap = max_threads(mt * nt, asym);
    while (waves > 1 && (waves * mt * nt > 64 || waves * 64 > plain_cap)) --waves;
    // The fused gate|up layer needs gate and up tiles in one workgroup.
    if (ydt == YDT_SILU_E4M3 && nt == 1) nt = 2;
    const int thread_cap = max_threads(mt * nt, asym, ydt == YDT_SILU_E4M3 && mt == 2 && nt == 2);
    while (waves > 1 && (waves * mt * nt > 64 || waves * 64 > thread_cap)) --waves;
    if (waves < 1 || waves > 16 || waves * mt * nt > 64 || waves * 64 > thread_cap) return false;
    // the form that quantizes its own input is built for one or two bands: fewer bands, the same split of K
    if (xq != 0 && nt > 2) {
        if (!auto_nt) return false;
        nt = 2;
    }
    const bool deep_built = mt == 1 && nt == 1 && xq == 0 && (ydt == (int)W4A8_BF16 || ydt == (int)W4A8_F32) && mode == MODE_CODE_EXACT;
    if (depth == 0) depth = (long_rows && deep_built) ? 4 : 2;   // elsewhere deeper rings cost occupancy and measured no faster
    return depth == 2 || (depth == 4 && deep_built);
}

int launch_linear_skinny(const uint8_t* x8, int64_t M, int64_t K, int64_t ldx8, const float* s_x,
                         const uint8_t* packed, const float* scales, int64_t N, int32_t G, void* y, w4a8_dtype ydt,
                         int64_t ldy, int nt, int waves, int depth, const float* w_out, int per_channel, int mode,
                         const float* y_scale, hipStream_t st, int xq, uint8_t* x8_out) {
    if (M < 1 || M > 64) return W4A8_ERR_SHAPE;
    if (xq != 0 && (M > 16 || M * K > 65536 || mode != MODE_CODE_EXACT)) return W4A8_ERR_SHAPE;
    const int C = (int)(K / 128), cpg = G / 128, NG = (int)(K / G);
    const int n_tiles = (int)((N + 15) / 16);
    const int mt = (M <= 16) ? 1 : (M <= 32) ? 2 : 4;
    if (!skinny_launch_shape(M, K, N, (int)ydt, mode, xq, nt, waves, depth)) return W4A8_ERR_SHAPE;
    const LinearArgs a{x8, (int)M, ldx8, s_x, packed, scales, (int)N, n_tiles, C, cpg, NG, y, ldy, w_out, per_channel, mode, y_scale,
                       xq, x8_out};
    if ((int)ydt == YDT_E4M3) {
        if (mode != MODE_CODE_EXACT || !y_scale) return W4A8_ERR_DTYPE;
        return launch_mt<uint8_t>(a, mt, nt, depth, waves, st);
    }
    if ((int)ydt == YDT_SILU_E4M3) {                             // pairs of gate and up tiles: nt is even here
        if (mode != MODE_CODE_EXACT || !y_scale || nt % 2 != 0) return W4A8_ERR_DTYPE;
        return launch_mt<SiluFp8>(a, mt, nt, depth, waves, st);
    }
    if (ydt == W4A8_F32) return launch_mt<float>(a, mt, nt, depth, waves, st);
    return launch_mt<uint16_t>(a, mt, nt, depth, waves, st);
}

}  // namespace w4a8
