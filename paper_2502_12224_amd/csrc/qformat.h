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
    static constexpr float OFF_BF16 = 136.f;   // 128 + 8
    static constexpr float OFF_F16 = 1032.f;   // 1024 + 8
};
template <>
struct QFmt<8> {
    static constexpr int KT = 32;
    static constexpr int NP = 8;
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
