// Device-side helpers shared by the W4A8 kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace w4a8 {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

// Saturate to the E4M3 range (Sec. 4.1: +-448) before the hardware rounding; NaN passes through.
__device__ __forceinline__ float sat448(float t) {
    const float c = __builtin_fminf(__builtin_fmaxf(t, -448.0f), 448.0f);
    return (t != t) ? t : c;
}

// Two float32 -> two E4M3 bytes (round to nearest even, saturating) in the low or high half of `old`.
__device__ __forceinline__ uint32_t cvt2(float a, float b, uint32_t old, bool high) {
    return high ? (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(sat448(a), sat448(b), (int)old, true)
                : (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(sat448(a), sat448(b), (int)old, false);
}

// ---------------------------------------------------------------------------------------------
// INT4 -> E4M3 (Eq. 10 with zero-point 0; the group scale is applied to the group's partial sum).
//   value   0    1    2    3    4    5    6    7     |  -8   -7   -6   -5   -4   -3   -2   -1
//   E4M3   00   38   40   44   48   4A   4C   4E     |  D0   CE   CC   CA   C8   C4   C0   B8
//
// Tiled layout: sign-magnitude nibbles, bit 3 = sign, bits 0..2 = |value| for values in [-7, 7]; -8 is stored as 1000.
// The E4M3 byte is then sign << 7 | table[magnitude]: one 8-entry table (one v_perm_b32 per four weights) and one
// and-or, four ALU ops per four weights.  1000 comes out of that as 0x80 (minus zero) and needs a fix-up to 0xD0;
// the packer marks every (row, group) that holds a -8 in the sign bit of the group's scale, so that the kernels
// run the fix-up only on chunks where a wavefront sees a marked scale.
//
// Canonical layout: two's-complement nibbles; the value is l when b3 = 0 and l - 8 when b3 = 1 (l = low three bits),
// each case an 8-entry table and a third v_perm_b32 to pick, byte by byte, the table that b3 names.
// ---------------------------------------------------------------------------------------------
// E4M3 bytes of the four sign-magnitude nibbles at bit offset SHIFT (0: low nibbles, 4: high nibbles) of the bytes
// of w, exact for every pattern except 1000, which gives 0x80.
template <int SHIFT>
__device__ __forceinline__ uint32_t sm_half_to_e4m3_fast(uint32_t w) {
    const uint32_t MAG_LO = 0x44403800u, MAG_HI = 0x4E4C4A48u;   // magnitudes 0..3, 4..7
    const uint32_t sel = (w >> SHIFT) & 0x07070707u;
    // v_perm_b32(S0, S1, sel): selector 0..3 -> bytes of S1, 4..7 -> bytes of S0
    const uint32_t mag = __builtin_amdgcn_perm(MAG_HI, MAG_LO, sel);
    const uint32_t sign = SHIFT ? w : (w << 4);
    return (sign & 0x80808080u) | mag;
}

// Turns every byte 0x80 of four E4M3 bytes produced by sm_half_to_e4m3_fast into 0xD0 (-8).
__device__ __forceinline__ uint32_t sm_fix_minus_eight(uint32_t e) {
    const uint32_t t = e ^ 0x80808080u;                          // zero exactly in the bytes to fix
    // zero-byte detector; exact here because a byte 0x01 cannot occur in t (0x81 is no output of the table)
    const uint32_t z = (t - 0x01010101u) & ~t & 0x80808080u;
    return e | (z >> 1) | (z >> 3);                              // 0x40 | 0x10 on top of the 0x80
}

template <int SHIFT>
__device__ __forceinline__ uint32_t sm_half_to_e4m3(uint32_t w) { return sm_fix_minus_eight(sm_half_to_e4m3_fast<SHIFT>(w)); }

// The 16 bytes (four dwords) of one tiled-layout slot -> the 32 operand bytes of one lane, in the order the
// layout defines: operand byte p (0..31) belongs to k = 32*kq + p.  ANY_M8 = false skips the -8 fix-up.
template <bool ANY_M8>
__device__ __forceinline__ v8i slot_to_operand(uint4 s) {
    const uint32_t w[4] = {s.x, s.y, s.z, s.w};
    v8i v;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        v[2 * d] = (int)(ANY_M8 ? sm_half_to_e4m3<0>(w[d]) : sm_half_to_e4m3_fast<0>(w[d]));
        v[2 * d + 1] = (int)(ANY_M8 ? sm_half_to_e4m3<4>(w[d]) : sm_half_to_e4m3_fast<4>(w[d]));
    }
    return v;
}

// Canonical layout: one dword holds eight two's-complement nibbles.  `lo` receives the E4M3 bytes of nibbles
// 0,2,4,6 (the low nibble of bytes 0..3), `hi` those of nibbles 1,3,5,7 (the high nibbles).
__device__ __forceinline__ void nibbles_to_e4m3(uint32_t w, uint32_t& lo, uint32_t& hi) {
    const uint32_t POS_LO = 0x44403800u, POS_HI = 0x4E4C4A48u;   // values 0..3, 4..7
    const uint32_t NEG_LO = 0xCACCCED0u, NEG_HI = 0xB8C0C4C8u;   // values -8..-5, -4..-1
    const uint32_t sel_l = w & 0x07070707u;
    const uint32_t sel_h = (w >> 4) & 0x07070707u;
    const uint32_t pos_l = __builtin_amdgcn_perm(POS_HI, POS_LO, sel_l);
    const uint32_t neg_l = __builtin_amdgcn_perm(NEG_HI, NEG_LO, sel_l);
    const uint32_t pos_h = __builtin_amdgcn_perm(POS_HI, POS_LO, sel_h);
    const uint32_t neg_h = __builtin_amdgcn_perm(NEG_HI, NEG_LO, sel_h);
    // byte i of the result = byte i of pos (selector i) or of neg (selector i + 4)
    const uint32_t mix_l = ((w >> 1) & 0x04040404u) | 0x03020100u;
    const uint32_t mix_h = ((w >> 5) & 0x04040404u) | 0x03020100u;
    lo = __builtin_amdgcn_perm(neg_l, pos_l, mix_l);
    hi = __builtin_amdgcn_perm(neg_h, pos_h, mix_h);
}

// ---------------------------------------------------------------------------------------------
// Two-level mode (Eq. 6-11 read literally): the FP8 weight is nearest_E4M3(code * s8), s8 the group's scale in the FP8
// domain.  nearest_E4M3 is odd, so the byte is sign << 7 | nearest_E4M3(|code| * |s8|): per (lane, chunk) a table of
// the nine magnitudes 0..8 times |s8| (float32 products, clamped to 448, rounded by the hardware converter), looked up
// exactly like the constant table of the code-exact mode.
// ---------------------------------------------------------------------------------------------
struct MagTable {
    uint32_t lo, hi;      // bytes: nearest_E4M3(m * |s8|) for m = 0..3 and m = 4..7
    uint32_t m8;          // the same for m = 8, in the low byte
};

__device__ __forceinline__ MagTable two_level_table(float s8) {
    const float a = fabsf(s8);
    auto c = [&](float m) { const float v = m * a; return v > 448.0f ? 448.0f : v; };   // a NaN scale stays NaN
    MagTable t;
    t.lo = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(0.0f, c(1.0f), 0, false);
    t.lo = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(c(2.0f), c(3.0f), (int)t.lo, true);
    t.hi = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(c(4.0f), c(5.0f), 0, false);
    t.hi = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(c(6.0f), c(7.0f), (int)t.hi, true);
    t.m8 = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(c(8.0f), 0.0f, 0, false) & 0xFFu;
    return t;
}

// E4M3 bytes of the four sign-magnitude nibbles at bit offset SHIFT of the bytes of w under table t; the pattern 1000
// (-8) comes out as 0x80 | t[0] and is put right by two_level_fix_minus_eight.
template <int SHIFT>
__device__ __forceinline__ uint32_t two_level_half_fast(uint32_t w, const MagTable& t) {
    const uint32_t sel = (w >> SHIFT) & 0x07070707u;
    const uint32_t mag = __builtin_amdgcn_perm(t.hi, t.lo, sel);
    const uint32_t sign = SHIFT ? w : (w << 4);
    return (sign & 0x80808080u) | mag;
}

template <int SHIFT>
__device__ __forceinline__ uint32_t two_level_fix_minus_eight(uint32_t e, uint32_t w, const MagTable& t) {
    const uint32_t x = ((w >> SHIFT) & 0x0F0F0F0Fu) ^ 0x08080808u;                   // zero bytes: nibble 1000
    const uint32_t z = ~(((x & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | x | 0x7F7F7F7Fu);       // 0x80 there, exact
    return e | ((z >> 7) * t.m8);                                                    // m8 < 0x80: no carries
}

template <bool ANY_M8>
__device__ __forceinline__ v8i slot_to_operand_two_level(uint4 s, const MagTable& t) {
    const uint32_t w[4] = {s.x, s.y, s.z, s.w};
    v8i v;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        uint32_t a = two_level_half_fast<0>(w[d], t), b = two_level_half_fast<4>(w[d], t);
        if (ANY_M8) {
            a = two_level_fix_minus_eight<0>(a, w[d], t);
            b = two_level_fix_minus_eight<4>(b, w[d], t);
        }
        v[2 * d] = (int)a;
        v[2 * d + 1] = (int)b;
    }
    return v;
}

// ---------------------------------------------------------------------------------------------
// Asymmetric format (Eq. 1 with unsigned codes 0..15, Eq. 8-9, Eq. 14): the weight is the integer u - z (code minus
// zero-point), in [-15, 15].  The stored nibble writes the code as u = 7.5 + h, h = +-(m + 0.5): bit 3 = 1 for codes
// 0..7 (m = 7 - u), bits 0..2 = m (codes 8..15: m = u - 8).  Two ways to the product, both exact in the operand:
//   - the MFMA-tiled kernel feeds nearest_E4M3(u - z), exact in E4M3.  The zero-point belongs to a (row, group), that
//     is to a lane for the length of a chunk: per (lane, chunk) a 16-entry table indexed by the nibble (sixteen float32
//     differences, rounded by the hardware converter, which is exact on them), an 8-entry lookup for each half of the
//     table and a third v_perm_b32 that picks, byte by byte, the half that bit 3 names;
//   - the skinny kernel feeds the half-integer h itself -- all sixteen values +-0.5 .. +-7.5 are exact in E4M3 and
//     the nibble is their sign-magnitude form, so the expansion is the signed format's short one, with no special
//     pattern -- and adds (7.5 - z) * sum_k x per chunk, the sum coming from one more MFMA against an operand of ones.
// ---------------------------------------------------------------------------------------------
struct AsymTable {
    uint32_t t[4];        // byte p % 4 of t[p / 4] = nearest_E4M3(code(p) - z) for nibble p
};

__device__ __forceinline__ AsymTable asym_table(uint32_t z) {
    const float zf = (float)(z & 15u);
    AsymTable T;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        // nibbles 4w .. 4w+3: codes 8 + p for p < 8, 15 - p for p >= 8
        const float c0 = (float)(w < 2 ? 8 + 4 * w : 15 - 4 * w), step = w < 2 ? 1.0f : -1.0f;
        int r = __builtin_amdgcn_cvt_pk_fp8_f32(c0 - zf, c0 + step - zf, 0, false);
        r = __builtin_amdgcn_cvt_pk_fp8_f32(c0 + 2.0f * step - zf, c0 + 3.0f * step - zf, r, true);
        T.t[w] = (uint32_t)r;
    }
    return T;
}

// The same table for the two-level reading of the asymmetric format (Eq. 10 taken literally with a zero-point): byte
// p = nearest_E4M3( float32(code(p) - z) * s8 ), the product one float32 multiplication, saturating at +-448.
__device__ __forceinline__ AsymTable asym_two_level_table(uint32_t z, float s8) {
    const float zf = (float)(z & 15u);
    AsymTable T;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const float c0 = (float)(w < 2 ? 8 + 4 * w : 15 - 4 * w), step = w < 2 ? 1.0f : -1.0f;
        T.t[w] = cvt2((c0 - zf) * s8, (c0 + step - zf) * s8, 0u, false);
        T.t[w] = cvt2((c0 + 2.0f * step - zf) * s8, (c0 + 3.0f * step - zf) * s8, T.t[w], true);
    }
    return T;
}

// E4M3 bytes of the half-integers h = +-(m + 0.5) of the four nibbles at bit offset SHIFT of the bytes of w.
template <int SHIFT>
__device__ __forceinline__ uint32_t asym_half_offset(uint32_t w) {
    const uint32_t MAG_LO = 0x46423C30u, MAG_HI = 0x4F4D4B49u;   // 0.5 1.5 2.5 3.5, 4.5 5.5 6.5 7.5
    const uint32_t sel = (w >> SHIFT) & 0x07070707u;
    const uint32_t mag = __builtin_amdgcn_perm(MAG_HI, MAG_LO, sel);
    const uint32_t sign = SHIFT ? w : (w << 4);
    return (sign & 0x80808080u) | mag;
}

__device__ __forceinline__ v8i slot_to_operand_half_offset(uint4 s) {
    const uint32_t w[4] = {s.x, s.y, s.z, s.w};
    v8i v;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        v[2 * d] = (int)asym_half_offset<0>(w[d]);
        v[2 * d + 1] = (int)asym_half_offset<4>(w[d]);
    }
    return v;
}

// E4M3 bytes of code - zero_point of the four nibbles at bit offset SHIFT (0: low nibbles, 4: high nibbles) of the
// bytes of w.
template <int SHIFT>
__device__ __forceinline__ uint32_t asym_half(uint32_t w, const AsymTable& T) {
    const uint32_t v = SHIFT ? (w >> 4) : w;
    const uint32_t sel = v & 0x07070707u;
    const uint32_t lo = __builtin_amdgcn_perm(T.t[1], T.t[0], sel);          // entries 0..7
    const uint32_t hi = __builtin_amdgcn_perm(T.t[3], T.t[2], sel);          // entries 8..15
    const uint32_t mix = ((v >> 1) & 0x04040404u) | 0x03020100u;             // byte i: selector i (lo) or i + 4 (hi)
    return __builtin_amdgcn_perm(hi, lo, mix);
}

__device__ __forceinline__ v8i slot_to_operand_asym(uint4 s, const AsymTable& T) {
    const uint32_t w[4] = {s.x, s.y, s.z, s.w};
    v8i v;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        v[2 * d] = (int)asym_half<0>(w[d], T);
        v[2 * d + 1] = (int)asym_half<4>(w[d], T);
    }
    return v;
}

// Bytes per (16-row band, group) record of the asymmetric format's parameters: 16 float32 scales, 16 zero-point bytes.
constexpr int ASYM_RECORD_BYTES = 80;

// True when some lane of the wavefront holds a scale whose sign bit is set (the packer's "-8 in this group" mark).
__device__ __forceinline__ bool any_marked(float s) { return __builtin_amdgcn_ballot_w64(__float_as_int(s) < 0) != 0; }

// D = A(16 x 128, E4M3) * B(128 x 16, E4M3) + C on the FP8 matrix unit, fp32 accumulation.
// Lane l carries row (A) / column (B) l % 16 and the 32 contraction positions 32*(l/16) .. +31; the result
// lane l carries column l % 16 and rows 4*(l/16) .. +3.
__device__ __forceinline__ v4f mfma_16x16x128_e4m3(v8i a, v8i b, v4f c) {
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0 /*A: E4M3*/, 0 /*B: E4M3*/, 0, 0, 0, 0);
}

// The same with block scales (the scaled form of the instruction): every lane supplies one E8M0 byte (2^(byte - 127))
// per operand for its 32 contraction positions, and the matrix unit multiplies each 32-deep partial sum by
// 2^(scale_a - 127) * 2^(scale_b - 127) before adding it up -- the power-of-two group scale of a weight band applied
// inside the instruction (Sec. 2.2: power-of-two scaling factors turn scaling into an exponent adjustment).
__device__ __forceinline__ v4f mfma_16x16x128_e4m3_scaled(v8i a, v8i b, v4f c, int scale_a, int scale_b) {
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0 /*A: E4M3*/, 0 /*B: E4M3*/, 0 /*byte 0*/, scale_a,
                                                            0 /*byte 0*/, scale_b);
}

constexpr int E8M0_ONE = 127;
// E8M0 byte of a float32 power of two: its exponent field (a mantissa, and the sign, are ignored).
__device__ __forceinline__ int e8m0_of(float s) { return (int)((__float_as_uint(s) >> 23) & 0xFFu); }

// Global memory -> LDS without staging registers: each lane copies 16 (4) bytes from base + offset (base
// wave-uniform, offset per lane) to LDS byte address lds_addr + 16 (4) * lane (lds_addr wave-uniform).  Written as
// assembly so that the compiler's wait-count pass does not treat the copy as an LDS store that every later LDS read
// might alias (it would wait for the just-issued prefetch before each read).  The caller orders a copy against its
// readers with lds_dma_wait_all() (plus a workgroup barrier when other wavefronts read the data), and against earlier
// reads of the destination with the `after` argument: a value obtained from those reads, which the copy waits for.
// The statements declare M0 as clobbered, so the compiler keeps no value of its own there across them.
__device__ __forceinline__ void lds_dma_16(const uint8_t* base, uint32_t offset, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(offset), "s"(base), "s"(lds_addr)
                 : "memory", "m0");
}
__device__ __forceinline__ void lds_dma_16_after(const uint8_t* base, uint32_t offset, uint32_t lds_addr, uint32_t after) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(offset), "s"(base), "s"(lds_addr), "v"(after)
                 : "memory", "m0");
}
__device__ __forceinline__ void lds_dma_4(const uint8_t* base, uint32_t offset, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :
                 : "v"(offset), "s"(base), "s"(lds_addr)
                 : "memory", "m0");
}

// Waits until every outstanding global load of this wavefront, the copies above included, has completed.
__device__ __forceinline__ void lds_dma_wait_all() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Marks the point in program order at which the four values must have been computed: an empty statement the
// compiler can neither move code across nor sink the producers of `v` below.  Emits no instruction.
__device__ __forceinline__ void keep_here(v4f& v) {
    asm volatile("" : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]));
}

__device__ __forceinline__ void keep_here(uint32_t& a, uint32_t& b) { asm volatile("" : "+v"(a), "+v"(b)); }
__device__ __forceinline__ void keep_here(uint32_t& a) { asm volatile("" : "+v"(a)); }

// float32 -> bf16 bits, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    const uint32_t u = __float_as_uint(f);
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    const uint32_t quiet = (u >> 16) | 0x0040u;
    return (uint16_t)(((u & 0x7FFFFFFFu) > 0x7F800000u) ? quiet : rounded);     // a select, not a branch
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Eq. 13 for one value: nearest_E4M3(x / s), the quotient one IEEE float32 division.
__device__ __forceinline__ uint8_t quantize_one(float x, float s) { return (uint8_t)(cvt2(x / s, 0.0f, 0u, false) & 0xFFu); }

// Eq. 13 for four values (IEEE float32 divisions, then one rounding onto the E4M3 grid), and the loaders that turn 16
// consecutive float32 / bf16 activations into floats.
__device__ __forceinline__ uint32_t quant4(float a, float b, float c, float d, float s) {
    // IEEE float32 division (correctly rounded), then one rounding onto the E4M3 grid
    uint32_t r = cvt2(a / s, b / s, 0u, false);
    return cvt2(c / s, d / s, r, true);
}

template <typename InT> struct Load16;   // 16 consecutive elements -> 16 floats
template <> struct Load16<float> {
    static __device__ __forceinline__ void load(const float* p, float (&v)[16]) {
        const float4* q = reinterpret_cast<const float4*>(p);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 t = q[i];
            v[4 * i] = t.x; v[4 * i + 1] = t.y; v[4 * i + 2] = t.z; v[4 * i + 3] = t.w;
        }
    }
    static __device__ __forceinline__ float one(const float* p) { return *p; }
};
template <> struct Load16<uint16_t> {
    static __device__ __forceinline__ void load(const uint16_t* p, float (&v)[16]) {
        const uint4* q = reinterpret_cast<const uint4*>(p);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint4 t = q[i];
            const uint32_t w[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[8 * i + 2 * j] = __uint_as_float(w[j] << 16);
                v[8 * i + 2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
            }
        }
    }
    static __device__ __forceinline__ float one(const uint16_t* p) { return bf16_bits_to_f32(*p); }
};

// silu(gate) * up in float32 (the decoder block's elementwise step): silu(g) = g / (1 + exp(-g)).
__device__ __forceinline__ float silu_mul_f32(float g, float u) { return g / (1.0f + expf(-g)) * u; }

// Output kinds of the linear kernels.  float, uint16_t (bf16) and uint8_t (E4M3 of the bf16 value, Eq. 13 with the next
// layer's scale) are what they say.  SiluFp8 is the gate|up layer of a decoder block with SiLU*mul and the down
// projection's activation quantization folded in: the weight rows come interleaved in 16-row bands (band 2p = gate
// rows 16p .. 16p+15, band 2p+1 = up rows 16p .. 16p+15), the kernel forms the bf16 values of both, and writes
// h8[m, 16p + i] = nearest_E4M3( bf16(silu(gate) * up) / scale ) -- N / 2 bytes per token.
struct SiluFp8 {
    uint8_t byte;
};
template <typename T> struct OutKind {
    using Slab = T;                        // what the epilogue holds per output channel before storing
    static constexpr bool SILU = false;
};
template <> struct OutKind<SiluFp8> {
    using Slab = uint16_t;
    static constexpr bool SILU = true;
};

// Output conversions of the linear kernels.  `q` is the static scale of the NEXT layer's activation quantization and
// counts only for FP8 output (uint8_t): the value is rounded to bf16 first, then quantized by Eq. 13, which is exactly
// what a bf16 output followed by the activation-quantize kernel produces.
template <typename T> struct OutCast;
template <> struct OutCast<float> {
    static __device__ __forceinline__ float cast(float v, float) { return v; }
};
template <> struct OutCast<uint16_t> {
    static __device__ __forceinline__ uint16_t cast(float v, float) { return f32_to_bf16_bits(v); }
};
template <> struct OutCast<uint8_t> {
    static __device__ __forceinline__ uint8_t cast(float v, float q) {
        return quantize_one(bf16_bits_to_f32(f32_to_bf16_bits(v)), q);
    }
};

}  // namespace w4a8
