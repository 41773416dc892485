// Device-native quantised weight layout and in-register dequantisation.
//
// A weight matrix [rows, K] is cut into 1 KiB tiles of 32 rows x KT columns
// (KT = 64 for int4, 32 for int8), tile (rb, kb) stored at tile index
// rb*(K/KT) + kb.  Inside a tile lane l = half*32 + n of a wavefront owns 16
// bytes: row rb*32 + n, columns kb*KT + half*(KT/2) + [0, KT/2).
//
//   int4: the lane's 32 codes sit in 4 dwords of 8; in dword d the code of
//         column 8d + 2i is nibble i and that of column 8d + 2i + 1 is nibble
//         i + 4 (unsigned nibble u = q + 8), so (dword >> 4i) & 0x000f000f
//         isolates one pair of neighbouring columns in the low bits of the
//         two 16-bit halves.
//   int8: 16 bytes in column order, offset binary u = q + 128.
//   int2: KT = 128; the lane's 64 codes sit in 4 dwords of 16; in dword d the
//         field (u in 0..3, signed code q = 2u - 3) of column 16d + 2i is bits
//         2i..2i+1 and that of column 16d + 2i + 1 is bits 16+2i..16+2i+1, so
//         (dword >> 8j) & (3 << 2i) isolates a pair of neighbouring columns in
//         the two 16-bit halves at four mantissa positions.
//
// A pair of codes becomes a pair of 16-bit floats by OR-ing the integer into
// the mantissa of a power of two: bf16 0x4300|u = 128 + u, fp16 0x6400|u =
// 1024 + u (exact).  Dot products therefore run on (u + C) and the constant
// is removed afterwards with the sum of the activations of the group:
//   sum x*q = sum x*(u + C) - (C + zero) * sum x.
#pragma once
#include "common.h"

namespace fate {

template <int BITS>
struct QFmt;
template <>
struct QFmt<4> {
    static constexpr int KT = 64;       // columns per tile
    static constexpr int NP = 16;       // 16-bit pairs per lane per tile
    static constexpr int MSTEPS = 4;    // 8-code matrix-core operands per lane per tile
    static constexpr float OFF_BF16 = 136.f;   // 128 + 8
    static constexpr float OFF_F16 = 1032.f;   // 1024 + 8
};
template <>
struct QFmt<2> {
    static constexpr int KT = 128;
    static constexpr int NP = 32;
    static constexpr int MSTEPS = 8;
    static constexpr float OFF_BF16 = 0.f;     // (the pair form is not used for this width)
    static constexpr float OFF_F16 = 0.f;
};
template <>
struct QFmt<8> {
    static constexpr int KT = 32;
    static constexpr int NP = 8;
    static constexpr int MSTEPS = 2;
    static constexpr float OFF_BF16 = 128.f;   // value is u itself
    static constexpr float OFF_F16 = 1152.f;   // 1024 + 128
};

#ifdef __HIPCC__
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;

// raw 16 bytes of one lane -> NP dwords, each a pair of bf16 (ACT_F16 = false)
// or fp16 (true) values (u + C) for two neighbouring columns.
template <int BITS, bool ACT_F16>
__device__ __forceinline__ void unpack_pairs(const uint4& raw, uint32_t* p) {
    const uint32_t r[4] = {raw.x, raw.y, raw.z, raw.w};
    if constexpr (BITS == 4) {
        const uint32_t magic = ACT_F16 ? 0x64006400u : 0x43004300u;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
#pragma unroll
            for (int i = 0; i < 4; ++i) p[4 * d + i] = ((r[d] >> (4 * i)) & 0x000f000fu) | magic;
        }
    } else {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            if constexpr (ACT_F16) {
                // bytes b0..b3 -> (0x6400|b0, 0x6400|b1), (0x6400|b2, 0x6400|b3)
                p[2 * d + 0] = __builtin_amdgcn_perm(0x64646464u, r[d], 0x04010400u);
                p[2 * d + 1] = __builtin_amdgcn_perm(0x64646464u, r[d], 0x04030402u);
            } else {
                // u <= 255 is exact in bf16: take the high half of float(u)
                uint32_t f0 = __float_as_uint((float)(r[d] & 0xffu));
                uint32_t f1 = __float_as_uint((float)((r[d] >> 8) & 0xffu));
                uint32_t f2 = __float_as_uint((float)((r[d] >> 16) & 0xffu));
                uint32_t f3 = __float_as_uint((float)(r[d] >> 24));
                p[2 * d + 0] = (f0 >> 16) | (f1 & 0xffff0000u);
                p[2 * d + 1] = (f2 >> 16) | (f3 & 0xffff0000u);
            }
        }
    }
}

typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;

// A constant the compiler must keep in a vector register.  (x & mask) | bits with two literal
// operands cannot be one VOP3 instruction on gfx9 (one scalar or literal operand per
// instruction), and the compiler then emits v_and + v_or and re-materialises the literals;
// with both constants in registers it selects v_and_or_b32.
__device__ __forceinline__ uint32_t vgpr_const(uint32_t c) {
    asm("" : "+v"(c));
    return c;
}
__device__ __forceinline__ uint32_t and_or_b32(uint32_t x, uint32_t mask, uint32_t bits) {
    return (x & vgpr_const(mask)) | vgpr_const(bits);
}

// raw 16 bytes of one lane -> MSTEPS operands of 8 fp16 values holding the
// signed codes q themselves (exact), in column order.  int4 uses two
// power-of-two mantissa tricks so that one shift serves four pairs:
// 0x6400|u = 1024 + u for nibbles at bits 0..3, 0x5400|(u << 4) = 64 + u for
// nibbles at bits 4..7 of each 16-bit half.
// One dword of sixteen 2-bit fields -> 16 fp16 values u (0..3) in column order: the field is
// OR-ed into the mantissa of 1024, 256, 64 or 16 by its bit position and the power of two
// is subtracted again (exact).
__device__ __forceinline__ void int2_fields_to_f16(uint32_t r, f16x2_t (&w)[8]) {
    const f16x2_t c0 = {(_Float16)1024.f, (_Float16)1024.f}, c1 = {(_Float16)256.f, (_Float16)256.f};
    const f16x2_t c2 = {(_Float16)64.f, (_Float16)64.f}, c3 = {(_Float16)16.f, (_Float16)16.f};
    const uint32_t hi = r >> 8;
    w[0] = __builtin_bit_cast(f16x2_t, and_or_b32(r, 0x00030003u, 0x64006400u)) - c0;
    w[1] = __builtin_bit_cast(f16x2_t, and_or_b32(r, 0x000c000cu, 0x5c005c00u)) - c1;
    w[2] = __builtin_bit_cast(f16x2_t, and_or_b32(r, 0x00300030u, 0x54005400u)) - c2;
    w[3] = __builtin_bit_cast(f16x2_t, and_or_b32(r, 0x00c000c0u, 0x4c004c00u)) - c3;
    w[4] = __builtin_bit_cast(f16x2_t, and_or_b32(hi, 0x00030003u, 0x64006400u)) - c0;
    w[5] = __builtin_bit_cast(f16x2_t, and_or_b32(hi, 0x000c000cu, 0x5c005c00u)) - c1;
    w[6] = __builtin_bit_cast(f16x2_t, and_or_b32(hi, 0x00300030u, 0x54005400u)) - c2;
    w[7] = __builtin_bit_cast(f16x2_t, and_or_b32(hi, 0x00c000c0u, 0x4c004c00u)) - c3;
}

template <int BITS>
__device__ __forceinline__ void codes_to_f16(const uint4& raw, f16x8_t* b) {
    const uint32_t r[4] = {raw.x, raw.y, raw.z, raw.w};
    if constexpr (BITS == 2) {
        const f16x2_t two = {(_Float16)2.f, (_Float16)2.f}, three = {(_Float16)3.f, (_Float16)3.f};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            f16x2_t w[8];
            int2_fields_to_f16(r[d], w);
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = w[i] * two - three;      // signed code 2u - 3, exact
            b[2 * d] = f16x8_t{w[0].x, w[0].y, w[1].x, w[1].y, w[2].x, w[2].y, w[3].x, w[3].y};
            b[2 * d + 1] = f16x8_t{w[4].x, w[4].y, w[5].x, w[5].y, w[6].x, w[6].y, w[7].x, w[7].y};
        }
    } else if constexpr (BITS == 4) {
        const f16x2_t offA = {(_Float16)1032.f, (_Float16)1032.f};   // 1024 + 8
        const f16x2_t offB = {(_Float16)72.f, (_Float16)72.f};       // 64 + 8
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t hi = r[d] >> 8;
            const f16x2_t w0 = __builtin_bit_cast(f16x2_t, and_or_b32(r[d], 0x000f000fu, 0x64006400u)) - offA;
            const f16x2_t w1 = __builtin_bit_cast(f16x2_t, and_or_b32(r[d], 0x00f000f0u, 0x54005400u)) - offB;
            const f16x2_t w2 = __builtin_bit_cast(f16x2_t, and_or_b32(hi, 0x000f000fu, 0x64006400u)) - offA;
            const f16x2_t w3 = __builtin_bit_cast(f16x2_t, and_or_b32(hi, 0x00f000f0u, 0x54005400u)) - offB;
            b[d] = f16x8_t{w0.x, w0.y, w1.x, w1.y, w2.x, w2.y, w3.x, w3.y};
        }
    } else {
        const f16x2_t off = {(_Float16)1152.f, (_Float16)1152.f};    // 1024 + 128
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            f16x2_t w[4];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const uint32_t v = r[2 * h + j];
                w[2 * j] = __builtin_bit_cast(f16x2_t, __builtin_amdgcn_perm(0x64646464u, v, 0x04010400u)) - off;
                w[2 * j + 1] = __builtin_bit_cast(f16x2_t, __builtin_amdgcn_perm(0x64646464u, v, 0x04030402u)) - off;
            }
            b[h] = f16x8_t{w[0].x, w[0].y, w[1].x, w[1].y, w[2].x, w[2].y, w[3].x, w[3].y};
        }
    }
}

template <bool ACT_F16>
__device__ __forceinline__ float dot2(uint32_t a, uint32_t w, float acc) {
    if constexpr (ACT_F16)
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, a), __builtin_bit_cast(f16x2_t, w), acc, false);
    else
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, w),
                                               acc, false);
}

template <int BITS, bool ACT_F16>
__device__ __forceinline__ constexpr float q_offset() {
    return ACT_F16 ? QFmt<BITS>::OFF_F16 : QFmt<BITS>::OFF_BF16;
}
#endif

}  // namespace fate
