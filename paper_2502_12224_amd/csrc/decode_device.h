// Device code shared by the decode-side FFN kernels: a register ring of
// weight tiles per wave and the matrix-core inner loop that consumes it.
//
// The multiply-adds run on the matrix cores although only 1..8 of the 32
// token columns of a 32x32x16 product are in use: widening the codes already
// takes most of the vector-ALU issue slots a wave has per byte streamed, and
// the matrix pipe runs beside it.  Operands: A = activations (fp16, a lane's
// row is a token, rows past the last token read a zero row in LDS), B = the
// lane's own 8 codes widened to fp16 integers (exact), so D[token][row] lands
// in the lane that owns the row's scale.  One accumulator per quantisation
// group, started from zero; the group's fp16 scale multiplies the fp32 group
// sum, so each weight enters exactly.
#pragma once
#include <hip/hip_fp16.h>
#include "common.h"
#include "qformat.h"

namespace fate {

constexpr int kTokPass = 8;    // tokens per pass over an expert's weights
constexpr int kLdsPad = 8;     // halves of padding per LDS activation row (bank spread)

// pointers into expert weights come out of a table in memory; telling the
// compiler they are global (not generic) pointers gives global_load, not flat_load
#if defined(__HIP_DEVICE_COMPILE__)
#define FATE_GLOBAL __attribute__((address_space(1)))
#else
#define FATE_GLOBAL
#endif
typedef const FATE_GLOBAL uint4* gu4_t;
typedef const FATE_GLOBAL uint16_t* gu16_t;
template <class T>
__device__ __forceinline__ const FATE_GLOBAL T* as_global(const void* p) {
    return (const FATE_GLOBAL T*)(uintptr_t)p;
}
__device__ __forceinline__ float half_bits_to_float(uint32_t b) {
    return __half2float(__ushort_as_half((unsigned short)b));
}

typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits
// for every outstanding global load of the wave, which would drain the ring
// of weight tiles that is meant to stay in flight across the barrier.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ f32x16_t f32x16_zero() {
    return f32x16_t{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
}

// bf16 x 8 -> fp16 x 8 (round to nearest even)
__device__ __forceinline__ uint4 bf16x8_to_f16x8(const uint4& v) {
    const uint32_t r[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const __half lo = __float2half_rn(bf16_lo(r[i]));
        const __half hi = __float2half_rn(bf16_hi(r[i]));
        o[i] = (uint32_t)__half_as_ushort(lo) | ((uint32_t)__half_as_ushort(hi) << 16);
    }
    return make_uint4(o[0], o[1], o[2], o[3]);
}

template <int NMAT, int D, int TPG, bool ZP = false>
struct TileRing {
    uint4 raw[NMAT][D];
    uint32_t sc[NMAT][D / TPG];   // fp16 bits of the group scale, one full register each
    uint32_t zr[NMAT][ZP ? D / TPG : 1];   // fp16 bits of the group zero-point (formats that have one)
};

// Zero-points, w = (u - z) * s: the matrix cores see the same symmetric codes q = a*u - c as
// without them, and the difference is one term per group,
//   sum_k (u_k - z) x_k = (sum_k q_k x_k + (c - a z) sum_k x_k) / a,
// with the group sums of the activations taken once per staged row.
template <int BITS> struct ZpFmt;
template <> struct ZpFmt<4> { static constexpr float inv_a = 1.0f, c_over_a = 8.0f; };     // q = u - 8
template <> struct ZpFmt<2> { static constexpr float inv_a = 0.5f, c_over_a = 1.5f; };     // q = 2u - 3
template <> struct ZpFmt<8> { static constexpr float inv_a = 1.0f, c_over_a = 128.0f; };   // not instantiated with zero-points

constexpr int kZpMaxGroups = 128;   // groups per staged activation row the zero-point path keeps sums for

// gs[t * G + g] = sum over group g of row t of the activations staged in LDS (fp16, row stride
// ldx halves); the whole workgroup calls it (256 threads), a quarter group per lane
__device__ __forceinline__ void stage_group_sums(const _Float16* xs, int ldx, int nt, int G, int group, float* gs) {
    const int tid = threadIdx.x;
    const int lim = nt * G * 4, q = group >> 2;
    for (int base = 0; base < lim; base += 256) {
        const int idx = base + tid;
        float s = 0.f;
        if (idx < lim) {
            const int tg = idx >> 2, t = tg / G, g = tg - t * G;
            const _Float16* p = xs + t * ldx + g * group + (idx & 3) * q;
            for (int c = 0; c < q; c += 8) {
                const f16x8_t v = *reinterpret_cast<const f16x8_t*>(p + c);
#pragma unroll
                for (int e = 0; e < 8; ++e) s += (float)v[e];
            }
        }
        s += __shfl_xor(s, 1);
        s += __shfl_xor(s, 2);
        if (idx < lim && (idx & 3) == 0) gs[idx >> 2] = s;
    }
}

// request the first D tiles of the groups [g_beg, g_end) (TPG tiles per group).
// sc[i]: this lane's row in the group-major scale array, srows = its row count;
// zp[i]: the same for the zero-points (read only if ZP).
template <int NMAT, int D, int TPG, bool ZP = false>
__device__ __forceinline__ void ring_start(TileRing<NMAT, D, TPG, ZP>& r, const gu4_t* wt, const gu16_t* sc,
                                           int srows, int g_beg, int g_end, const gu16_t* zp = nullptr) {
    const int tbeg = g_beg * TPG, tend = g_end * TPG;
#pragma unroll
    for (int j = 0; j < D; ++j) {
        if (tbeg + j < tend) {
#pragma unroll
            for (int i = 0; i < NMAT; ++i) {
                r.raw[i][j] = wt[i][(size_t)(tbeg + j) * 64];
                if (j % TPG == 0) {
                    r.sc[i][j / TPG] = sc[i][(size_t)(g_beg + j / TPG) * srows];
                    if constexpr (ZP) r.zr[i][j / TPG] = zp[i][(size_t)(g_beg + j / TPG) * srows];
                }
            }
        }
    }
}

// One wave accumulates, for the (up to 8) activation rows staged in LDS, the
// products with NMAT weight row-blocks over the groups [g_beg, g_end);
// ring_start must have been called with the same range.  xa: this lane's
// activation row in LDS (fp16), already offset by its half of a tile; its
// column 0 is absolute column k_base.  out[i][j]: row n of matrix i, token
// 4*half + j.  With ZP: zp as in ring_start, gs = the group sums of this lane's first token
// (token 4*half), rows gs_ld floats apart, its entry 0 being group g_off.
template <int BITS, int TPG, int NMAT, int D, bool ZP = false>
__device__ __forceinline__ void ring_run(TileRing<NMAT, D, TPG, ZP>& r, const gu4_t* wt, const gu16_t* sc,
                                         int srows, int g_beg, int g_end, const _Float16* xa, int k_base,
                                         float (&out)[NMAT][4], const gu16_t* zp = nullptr,
                                         const float* gs = nullptr, int gs_ld = 0, int g_off = 0) {
    constexpr int KT = QFmt<BITS>::KT, S = QFmt<BITS>::MSTEPS;
    static_assert(D % TPG == 0, "ring depth must hold whole groups");
    const int tbeg = g_beg * TPG, tend = g_end * TPG;
    const f32x16_t zero = f32x16_zero();
    for (int base = tbeg; base < tend; base += D) {
#pragma unroll
        for (int jg = 0; jg < D / TPG; ++jg) {
            if (base + jg * TPG < tend) {
                f32x16_t acc[NMAT];
                float s[NMAT];
#pragma unroll
                for (int i = 0; i < NMAT; ++i) s[i] = half_bits_to_float(r.sc[i][jg]);
                float dz[NMAT];
                if constexpr (ZP) {
#pragma unroll
                    for (int i = 0; i < NMAT; ++i) dz[i] = ZpFmt<BITS>::c_over_a - half_bits_to_float(r.zr[i][jg]);
                }
                const int gcur = base / TPG + jg;
                const int gnext = gcur + D / TPG;
                if (gnext < g_end) {
#pragma unroll
                    for (int i = 0; i < NMAT; ++i) {
                        r.sc[i][jg] = sc[i][(size_t)gnext * srows];
                        if constexpr (ZP) r.zr[i][jg] = zp[i][(size_t)gnext * srows];
                    }
                }
#pragma unroll
                for (int tl = 0; tl < TPG; ++tl) {
                    const int j = jg * TPG + tl;
                    const int tile = base + j;
                    const _Float16* xt = xa + (tile * KT - k_base);
                    f16x8_t av[S];
#pragma unroll
                    for (int st = 0; st < S; ++st) av[st] = *reinterpret_cast<const f16x8_t*>(xt + 8 * st);
#pragma unroll
                    for (int i = 0; i < NMAT; ++i) {
                        f16x8_t b[S];
                        codes_to_f16<BITS>(r.raw[i][j], b);
                        if (tile + D < tend) r.raw[i][j] = wt[i][(size_t)(tile + D) * 64];
#pragma unroll
                        for (int st = 0; st < S; ++st)
                            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                                av[st], b[st], (tl == 0 && st == 0) ? zero : acc[i], 0, 0, 0);
                    }
                }
                if constexpr (ZP) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float gsum = gs[j * gs_ld + (gcur - g_off)];
#pragma unroll
                        for (int i = 0; i < NMAT; ++i)
                            out[i][j] = fmaf(s[i], fmaf(ZpFmt<BITS>::inv_a, acc[i][j], dz[i] * gsum), out[i][j]);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < NMAT; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j) out[i][j] = fmaf(s[i], acc[i][j], out[i][j]);
                }
            }
        }
    }
}

// The register ring's type depends on the tiles per group; the format of an
// expert is only known at run time, so the kernels branch once to the matching
// instantiation.  tpg in {1, 2, 4} for int4, {2, 4} for int8, {1, 2} for int2 (checked on the host
// for the descriptor's widths, on the device for an expert entry of another width).
#define FATE_FORMAT_SWITCH(bits, tpg, BODY)                \
    if ((bits) == 4) {                                     \
        if ((tpg) == 2) { BODY(4, 2) }                     \
        else if ((tpg) == 1) { BODY(4, 1) }                \
        else { BODY(4, 4) }                                \
    } else {                                               \
        if ((tpg) == 4) { BODY(8, 4) }                     \
        else { BODY(8, 2) }                                \
    }

__host__ __device__ inline int tile_columns(int bits) { return bits == 4 ? 64 : (bits == 8 ? 32 : 128); }
// the same with the 2-bit format (the separate-call FFN kernels; the one-call layer keeps 4 / 8 bits)
#define FATE_FORMAT_SWITCH_ALL(bits, tpg, BODY)            \
    if ((bits) == 2) {                                     \
        if ((tpg) == 1) { BODY(2, 1) }                     \
        else { BODY(2, 2) }                                \
    } else {                                               \
        FATE_FORMAT_SWITCH(bits, tpg, BODY)                \
    }

// formats with zero-points: 4 and 2 bits
#define FATE_FORMAT_SWITCH_ZP(bits, tpg, BODY)             \
    if ((bits) == 2) {                                     \
        if ((tpg) == 1) { BODY(2, 1) }                     \
        else { BODY(2, 2) }                                \
    } else {                                               \
        if ((tpg) == 2) { BODY(4, 2) }                     \
        else if ((tpg) == 1) { BODY(4, 1) }                \
        else { BODY(4, 4) }                                \
    }

static inline bool decode_group_ok(int bits, int group) {
    if (group % tile_columns(bits)) return false;
    const int tpg = group / tile_columns(bits);
    if (bits == 2) return tpg == 1 || tpg == 2;
    return bits == 4 ? (tpg == 1 || tpg == 2 || tpg == 4) : (tpg == 2 || tpg == 4);
}

// An expert entry as the FFN kernels can read it: a width they know, a group that is a whole
// number of tiles and one of the instantiated tiles-per-group, dimensions that are whole groups.
__host__ __device__ inline bool entry_format_ok(int bits, int group, int H, int I) {
    if (bits != 2 && bits != 4 && bits != 8) return false;
    const int kt = tile_columns(bits);
    if (group <= 0 || group % kt || H % group || I % group) return false;
    const int tpg = group / kt;
    if (bits == 2) return tpg == 1 || tpg == 2;
    return bits == 4 ? (tpg == 1 || tpg == 2 || tpg == 4) : (tpg == 2 || tpg == 4);
}

// sigmoid(x . g) for one token row (bf16 inputs), one wave
__device__ __forceinline__ float wave_sigmoid_dot_bf16(const uint4* xr, const uint4* gv, int nvec) {
    const int lane = threadIdx.x & 63;
    float acc = 0.f;
    for (int c = lane; c < nvec; c += 64) {
        const uint4 xv = xr[c], g = gv[c];
        acc = fmaf(bf16_lo(xv.x), bf16_lo(g.x), acc); acc = fmaf(bf16_hi(xv.x), bf16_hi(g.x), acc);
        acc = fmaf(bf16_lo(xv.y), bf16_lo(g.y), acc); acc = fmaf(bf16_hi(xv.y), bf16_hi(g.y), acc);
        acc = fmaf(bf16_lo(xv.z), bf16_lo(g.z), acc); acc = fmaf(bf16_hi(xv.z), bf16_hi(g.z), acc);
        acc = fmaf(bf16_lo(xv.w), bf16_lo(g.w), acc); acc = fmaf(bf16_hi(xv.w), bf16_hi(g.w), acc);
    }
    acc = wave_sum(acc);
    return 1.0f / (1.0f + expf(-acc));
}

}  // namespace fate
