// Prefill-side expert FFN: MFMA grouped GEMM over quantised experts.
//
// Four launches per layer:
//   prep     x (bf16) -> fp16 copy, shared-expert gate values, and the tile
//            tables (prefix sums of tiles per expert segment) of both GEMMs;
//   up       grouped GEMM  h = silu(X W1^T) * (X W3^T)   -> fp16 [rows, I]
//   down     grouped GEMM  Yp = h W2^T                     -> fp16 [rows, H]
//   combine  y[t] = sum_j w[t,j] Yp[inv_perm[t*k+j]] + sum_s g_s(t) Yp_s[t]
// Rows are (token, expert) pairs in the sorted order of the permutation, so
// an expert's rows are contiguous; shared experts are extra segments of N rows.
//
// GEMM tile: a workgroup of four waves owns 64 rows x 128 weight rows; each
// wave owns 32 weight rows (one device-native tile row-block) and all 64
// rows; two workgroups share a compute unit (two waves per SIMD), so that one
// wave's dequantisation and LDS reads run under the other's matrix products
// (128-row tiles at one wave per SIMD left the matrix pipe idle 78 % of the time).  Activations go through LDS in chunks of 128 columns; weights go
// straight from global memory into registers in their tile layout (one
// contiguous KiB per wave load) and are dequantised there to fp16
// (exact code, one rounding in code*scale), which is the B operand of
// v_mfma_f32_32x32x16_f16.  Accumulation is fp32.
#include <hip/hip_fp16.h>
#include <algorithm>
#include "common.h"
#include "qformat.h"
#include "ffn_internal.h"

namespace fate {

typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2v_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kBMUp = 64;           // rows per workgroup tile of the up GEMM (two matrices)
constexpr int kBMDown = 64;         // rows per workgroup tile of the down GEMM
constexpr int kBN = 128;            // weight rows per workgroup tile (4 waves x 32)
constexpr int kKC = 128;            // columns per LDS chunk
constexpr int kLdsRow = kKC + 8;    // halves per LDS row (16-byte pad against bank conflicts)
constexpr int kWRing = 2;           // chunks of weights in flight per wave

// Workgroup barrier that orders LDS traffic only: __syncthreads() would also wait for the
// weight tiles that are meant to stay in flight across it.
__device__ __forceinline__ void lds_only_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

#if defined(__HIP_DEVICE_COMPILE__)
#define FATE_GLOBAL __attribute__((address_space(1)))
#else
#define FATE_GLOBAL
#endif
typedef const FATE_GLOBAL uint4* gu4p_t;
typedef const FATE_GLOBAL uint16_t* gu16p_t;

struct GemmArgs {
    const __half* A_r; int lda_r;      // activations fp16 of routed segments
    const __half* A_s; int lda_s;      // activations fp16 of shared segments
    int H;                             // hidden size
    int mode;                          // 0 = up (two matrices + SwiGLU, K = H), 1 = down (K = I of the expert)
    const fate_qexpert* experts; const fate_qexpert* shared;
    int E, n_shared, N, k;
    const int32_t* offsets; const int32_t* perm;
    const int32_t* tile_start;         // [E + n_shared + 1]
    __half* out_r; int ldo_r;          // routed rows, by sorted position
    __half* out_s; int ldo_s;          // shared rows, s*N + t
    int nb_r, nb_s;                    // column blocks per routed / shared segment
    int bits_r, group_r, bits_s, group_s;
    int32_t* status;
};

__global__ __launch_bounds__(256) void prefill_prep_kernel(const uint16_t* __restrict__ x, int N, int H, int E,
                                                           int n_shared, const int32_t* __restrict__ offsets,
                                                           const uint16_t* __restrict__ shared_gate,
                                                           __half* __restrict__ xh, float* __restrict__ sgate,
                                                           int32_t* __restrict__ tab_up,
                                                           int32_t* __restrict__ tab_down, int nb_r_up,
                                                           int nb_s_up, int nb_r_down, int nb_s_down, PartSel sel) {
    __shared__ float red[4];
    const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nvec = H >> 3;
    // (a later piece of a layer processed in pieces finds x and the gate values in place: only the tables change)
    if (sel.first) {
    const uint4* xr = reinterpret_cast<const uint4*>(x) + (size_t)t * nvec;
    uint4* xo = reinterpret_cast<uint4*>(xh) + (size_t)t * nvec;
    const uint4* gv = reinterpret_cast<const uint4*>(shared_gate);
    float acc = 0.f;
    for (int c = tid; c < nvec; c += 256) {
        const uint4 v = xr[c];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        uint32_t o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            __half2 h = __floats2half2_rn(bf16_lo(w[i]), bf16_hi(w[i]));
            o[i] = *reinterpret_cast<uint32_t*>(&h);
        }
        xo[c] = make_uint4(o[0], o[1], o[2], o[3]);
        if (gv) {
            const uint4 g = gv[c];
            const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc = fmaf(bf16_lo(w[i]), bf16_lo(gw[i]), acc);
                acc = fmaf(bf16_hi(w[i]), bf16_hi(gw[i]), acc);
            }
        }
    }
    if (gv) {
        acc = wave_sum(acc);
        if (lane == 0) red[wave] = acc;
        __syncthreads();
        if (tid == 0) sgate[t] = 1.0f / (1.0f + expf(-((red[0] + red[1]) + (red[2] + red[3]))));
    }
    }
    if (t == 0 && wave == 0) {
        // tile tables: exclusive prefix sums over the segments, 64 segments per step of one wave
        const int nseg = E + n_shared;
        int ru = 0, rd = 0;
        for (int s0 = 0; s0 < nseg; s0 += 64) {
            const int s = s0 + lane;
            int cu = 0, cd = 0;
            if (s < nseg) {
                // a piece holds the routed experts of its mask; the shared experts go with the first piece
                const bool mine = s < E ? ((sel.mask[s >> 6] >> (s & 63)) & 1ull) != 0 : sel.first != 0;
                const int T = !mine ? 0 : (s < E ? offsets[s + 1] - offsets[s] : N);
                cu = ((T + kBMUp - 1) / kBMUp) * (s < E ? nb_r_up : nb_s_up);
                cd = ((T + kBMDown - 1) / kBMDown) * (s < E ? nb_r_down : nb_s_down);
            }
            int iu = cu, id = cd;
#pragma unroll
            for (int sh = 1; sh < 64; sh <<= 1) {
                const int pu = __shfl_up(iu, sh, 64), pd = __shfl_up(id, sh, 64);
                if (lane >= sh) { iu += pu; id += pd; }
            }
            if (s < nseg) {
                tab_up[s] = ru + iu - cu;
                tab_down[s] = rd + id - cd;
            }
            ru += __shfl(iu, 63, 64);
            rd += __shfl(id, 63, 64);
        }
        if (lane == 0) {
            tab_up[nseg] = ru;
            tab_down[nseg] = rd;
        }
    }
}

// raw tile piece of one lane -> fp16 B operands (8 columns each)
template <int BITS>
__device__ __forceinline__ void dequant_tile(const uint4& raw, uint32_t scale_bits, f16x8_t* b) {
    const f16x2v_t s2 = {__builtin_bit_cast(_Float16, (unsigned short)scale_bits),
                         __builtin_bit_cast(_Float16, (unsigned short)scale_bits)};
    const uint32_t r[4] = {raw.x, raw.y, raw.z, raw.w};
    if constexpr (BITS == 2) {
        // sixteen fields per dword -> two operands of 8 columns; signed code 2u - 3 (exact), one rounding in code * scale
        const f16x2v_t two = {(_Float16)2.f, (_Float16)2.f}, three = {(_Float16)3.f, (_Float16)3.f};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            f16x2_t f[8];
            int2_fields_to_f16(r[d], f);
            f16x2v_t w[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = (__builtin_bit_cast(f16x2v_t, f[i]) * two - three) * s2;
            b[2 * d] = f16x8_t{w[0].x, w[0].y, w[1].x, w[1].y, w[2].x, w[2].y, w[3].x, w[3].y};
            b[2 * d + 1] = f16x8_t{w[4].x, w[4].y, w[5].x, w[5].y, w[6].x, w[6].y, w[7].x, w[7].y};
        }
    } else if constexpr (BITS == 4) {
        const f16x2v_t offA = {(_Float16)1032.f, (_Float16)1032.f};   // 1024 + 8
        const f16x2v_t offB = {(_Float16)72.f, (_Float16)72.f};       // 64 + 8
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t hi = r[d] >> 8;
            uint32_t u[4];
            u[0] = and_or_b32(r[d], 0x000f000fu, 0x64006400u);   // columns 0,1: 1024 + u
            u[1] = and_or_b32(r[d], 0x00f000f0u, 0x54005400u);   // columns 2,3: 64 + u
            u[2] = and_or_b32(hi, 0x000f000fu, 0x64006400u);     // columns 4,5
            u[3] = and_or_b32(hi, 0x00f000f0u, 0x54005400u);     // columns 6,7
            f16x2v_t w[4];
            w[0] = (__builtin_bit_cast(f16x2v_t, u[0]) - offA) * s2;
            w[1] = (__builtin_bit_cast(f16x2v_t, u[1]) - offB) * s2;
            w[2] = (__builtin_bit_cast(f16x2v_t, u[2]) - offA) * s2;
            w[3] = (__builtin_bit_cast(f16x2v_t, u[3]) - offB) * s2;
            b[d] = f16x8_t{w[0].x, w[0].y, w[1].x, w[1].y, w[2].x, w[2].y, w[3].x, w[3].y};
        }
    } else {
        const f16x2v_t off = {(_Float16)1152.f, (_Float16)1152.f};    // 1024 + 128
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            f16x2v_t w[4];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const uint32_t v = r[2 * h + j];
                const uint32_t p0 = __builtin_amdgcn_perm(0x64646464u, v, 0x04010400u);
                const uint32_t p1 = __builtin_amdgcn_perm(0x64646464u, v, 0x04030402u);
                w[2 * j] = (__builtin_bit_cast(f16x2v_t, p0) - off) * s2;
                w[2 * j + 1] = (__builtin_bit_cast(f16x2v_t, p1) - off) * s2;
            }
            b[h] = f16x8_t{w[0].x, w[0].y, w[1].x, w[1].y, w[2].x, w[2].y, w[3].x, w[3].y};
        }
    }
}

// the same with a zero-point: w = (u - z) * s on the unsigned field u (exact), two roundings
template <int BITS>
__device__ __forceinline__ void dequant_tile_zp(const uint4& raw, uint32_t scale_bits, uint32_t zero_bits, f16x8_t* b) {
    static_assert(BITS == 4 || BITS == 2, "zero-points come with the 4- and 2-bit formats");
    const f16x2v_t s2 = {__builtin_bit_cast(_Float16, (unsigned short)scale_bits),
                         __builtin_bit_cast(_Float16, (unsigned short)scale_bits)};
    const f16x2v_t z2 = {__builtin_bit_cast(_Float16, (unsigned short)zero_bits),
                         __builtin_bit_cast(_Float16, (unsigned short)zero_bits)};
    const uint32_t r[4] = {raw.x, raw.y, raw.z, raw.w};
    if constexpr (BITS == 2) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            f16x2_t f[8];
            int2_fields_to_f16(r[d], f);
            f16x2v_t w[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = (__builtin_bit_cast(f16x2v_t, f[i]) - z2) * s2;
            b[2 * d] = f16x8_t{w[0].x, w[0].y, w[1].x, w[1].y, w[2].x, w[2].y, w[3].x, w[3].y};
            b[2 * d + 1] = f16x8_t{w[4].x, w[4].y, w[5].x, w[5].y, w[6].x, w[6].y, w[7].x, w[7].y};
        }
    } else {
        const f16x2v_t cA = {(_Float16)1024.f, (_Float16)1024.f}, cB = {(_Float16)64.f, (_Float16)64.f};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t hi = r[d] >> 8;
            f16x2v_t w[4];
            w[0] = ((__builtin_bit_cast(f16x2v_t, and_or_b32(r[d], 0x000f000fu, 0x64006400u)) - cA) - z2) * s2;
            w[1] = ((__builtin_bit_cast(f16x2v_t, and_or_b32(r[d], 0x00f000f0u, 0x54005400u)) - cB) - z2) * s2;
            w[2] = ((__builtin_bit_cast(f16x2v_t, and_or_b32(hi, 0x000f000fu, 0x64006400u)) - cA) - z2) * s2;
            w[3] = ((__builtin_bit_cast(f16x2v_t, and_or_b32(hi, 0x00f000f0u, 0x54005400u)) - cB) - z2) * s2;
            b[d] = f16x8_t{w[0].x, w[0].y, w[1].x, w[1].y, w[2].x, w[2].y, w[3].x, w[3].y};
        }
    }
}

template <int BITS, int NMAT, int kBM, bool ZP = false>
__device__ __forceinline__ void gemm_tile(const GemmArgs& a, const fate_qexpert* ex, int group, int row0, int T,
                                          int nblk, const int* arow, __half* xt, __half* out, int ldo,
                                          int out_row0, int Nout, int K, const __half* A, int lda) {
    constexpr int KT = QFmt<BITS>::KT;
    constexpr int TPC = kKC / KT;          // weight tiles per chunk (1 | 2 | 4)
    constexpr int SPT = KT / 16;           // MFMA k-slots per tile (8 | 4 | 2)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, half = lane >> 5;
    const int G = K / group, tiles_k = K / KT, nchunk = K / kKC;
    const int wrow0 = nblk * kBN + wave * 32;              // first weight row of this wave
    const bool wlive = wrow0 < Nout;
    const int nmt = (min(kBM, T - row0) + 31) >> 5;        // 32-row tiles of this block that hold rows
    gu4p_t wt[NMAT];
    gu16p_t sc[NMAT];
    gu16p_t zp[NMAT];
    {
        const void* wp[2] = {a.mode == 0 ? ex->w1 : ex->w2, ex->w3};
        const void* sp[2] = {a.mode == 0 ? ex->s1 : ex->s2, ex->s3};
        const void* zq[2] = {a.mode == 0 ? ex->z1 : ex->z2, ex->z3};
#pragma unroll
        for (int i = 0; i < NMAT; ++i) {
            wt[i] = (gu4p_t)(uintptr_t)wp[i] + (size_t)(wrow0 >> 5) * tiles_k * 64 + lane;
            sc[i] = (gu16p_t)(uintptr_t)sp[i] + wrow0 + n;          // group-major scales: [G][Nout]
            zp[i] = (gu16p_t)(uintptr_t)(ZP ? zq[i] : sp[i]) + wrow0 + n;     // zero-points, same layout
        }
    }
    f32x16_t acc[NMAT][kBM / 32];
#pragma unroll
    for (int i = 0; i < NMAT; ++i)
#pragma unroll
        for (int mt = 0; mt < kBM / 32; ++mt)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[i][mt][j] = 0.f;

    // staging assignment: thread -> (row r0 + 16*i, 16-byte column piece cp)
    const int cp = tid & 15, r0 = tid >> 4;
    uint4 xr[kBM / 16];
    uint4 raw[kWRing][NMAT][TPC];
    uint32_t sbits[kWRing][NMAT][TPC];
    uint32_t zbits[ZP ? kWRing : 1][NMAT][TPC];
    // (the load is unconditional and the row is clamped: a branch around a load makes the
    // compiler wait for every outstanding load at the next use, which empties the weight ring)
    // the rows this thread stages do not change from chunk to chunk; a missing row reads row 0
    // and is masked to zero (an AND, not a select: a select lets the compiler put the load
    // back under a branch)
    uint32_t xoff[kBM / 16];       // element offsets (rows * lda < 2^31: checked by the entry point)
    uint32_t xmask[kBM / 16];
#pragma unroll
    for (int i = 0; i < kBM / 16; ++i) {
        const int ar = arow[r0 + 16 * i];
        xoff[i] = (uint32_t)(ar >= 0 ? ar : 0) * (uint32_t)lda + cp * 8;
        xmask[i] = ar >= 0 ? 0xffffffffu : 0u;
    }
    auto load_x = [&](int kc) {
#pragma unroll
        for (int i = 0; i < kBM / 16; ++i) {
            const uint4 v = *reinterpret_cast<const uint4*>(A + xoff[i] + kc * kKC);
            xr[i] = make_uint4(v.x & xmask[i], v.y & xmask[i], v.z & xmask[i], v.w & xmask[i]);
        }
    };
    auto request_w = [&](int u, int kc) {
#pragma unroll
        for (int i = 0; i < NMAT; ++i)
#pragma unroll
            for (int tl = 0; tl < TPC; ++tl) {
                const int tile = kc * TPC + tl;
                raw[u][i][tl] = wt[i][(size_t)tile * 64];
                sbits[u][i][tl] = sc[i][(size_t)((tile * KT) / group) * Nout];
                if constexpr (ZP) zbits[u][i][tl] = zp[i][(size_t)((tile * KT) / group) * Nout];
            }
    };
    auto dequant = [&](int u, int i, int tl, f16x8_t* b) {
        if constexpr (ZP) dequant_tile_zp<BITS>(raw[u][i][tl], sbits[u][i][tl], zbits[u][i][tl], b);
        else dequant_tile<BITS>(raw[u][i][tl], sbits[u][i][tl], b);
    };
    // two activation tiles in LDS: chunk kc is multiplied from tile kc & 1 while chunk kc + 1 is
    // written into the other one, so a chunk costs one barrier and a wave's dequantisation is
    // not fenced off from its matrix products
    auto stage_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kBM / 16; ++i)
            *reinterpret_cast<uint4*>(xt + buf * (kBM * kLdsRow) + (r0 + 16 * i) * kLdsRow + cp * 8) = xr[i];
    };
    auto multiply = [&](f16x8_t (&b)[NMAT][kKC / 16], int buf) {
        const __half* xb = xt + buf * (kBM * kLdsRow);
#pragma unroll
        for (int mt = 0; mt < kBM / 32; ++mt) {
            if (mt < nmt) {
#pragma unroll
                for (int tl = 0; tl < TPC; ++tl)
#pragma unroll
                    for (int d = 0; d < SPT; ++d) {
                        const int kl = tl * KT + half * (KT / 2) + 8 * d;
                        const f16x8_t av = *reinterpret_cast<const f16x8_t*>(xb + (mt * 32 + n) * kLdsRow + kl);
#pragma unroll
                        for (int i = 0; i < NMAT; ++i)
                            acc[i][mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, b[i][tl * SPT + d], acc[i][mt], 0, 0, 0);
                    }
            }
        }
    };
    // At the top of iteration kc: tile kc & 1 holds chunk kc (a barrier has passed since it was
    // written), xr holds chunk kc + 1, the weights of chunks kc .. kc + kWRing - 1 are requested.
    static_assert(kWRing == 2, "ring slot and LDS tile of a chunk are both kc & 1");
    int kc_done = 0;
    const bool steady = BITS == 4 && wlive && nchunk >= kWRing;
    // (int4 only: the int8 instantiation holds twice the tiles per chunk and has no registers
    // left for a second copy of the loop)
    if (steady) {
#pragma unroll
        for (int u = 0; u < kWRing; ++u) request_w(u, u);
    } else {
#pragma unroll
        for (int u = 0; u < kWRing; ++u)
            if (wlive && u < nchunk) request_w(u, u);
    }
    load_x(0);
    stage_x(0);
    load_x(min(1, nchunk - 1));
    lds_only_barrier();
    if (steady) {
        // Steady state without a branch around any load: weights kWRing chunks ahead, the
        // activations after next requested before the refill (loads return in order, and the
        // next iteration must not wait for that refill).  Near the end the requests are clamped
        // to the last chunk instead of being skipped: a few redundant loads, no branch.
        const int nfull = nchunk / kWRing * kWRing;
        for (int kc0 = 0; kc0 < nfull; kc0 += kWRing) {
#pragma unroll
            for (int u = 0; u < kWRing; ++u) {
                const int kc = kc0 + u;
                stage_x(u ^ 1);
                load_x(min(kc + 2, nchunk - 1));
                f16x8_t b[NMAT][kKC / 16];
#pragma unroll
                for (int i = 0; i < NMAT; ++i)
#pragma unroll
                    for (int tl = 0; tl < TPC; ++tl) dequant(u, i, tl, &b[i][tl * SPT]);
                request_w(u, min(kc + kWRing, nchunk - 1));
                multiply(b, u);
                lds_only_barrier();   // chunk kc + 1 is visible, everyone is done reading chunk kc
            }
        }
        kc_done = nfull;
    }
    // the last chunks (and shapes with a short K, or a wave without weight rows)
    for (int kc0 = kc_done; kc0 < nchunk; kc0 += kWRing) {
#pragma unroll
        for (int u = 0; u < kWRing; ++u) {
            const int kc = kc0 + u;
            if (kc < nchunk) {
                if (kc + 1 < nchunk) stage_x(u ^ 1);
                if (kc + 2 < nchunk) load_x(kc + 2);
                f16x8_t b[NMAT][kKC / 16];
                if (wlive) {
#pragma unroll
                    for (int i = 0; i < NMAT; ++i)
#pragma unroll
                        for (int tl = 0; tl < TPC; ++tl)
                            dequant(u, i, tl, &b[i][tl * SPT]);
                    if (kc + kWRing < nchunk) request_w(u, kc + kWRing);
                    multiply(b, u);
                }
                lds_only_barrier();
            }
        }
    }
    if (!wlive) return;
    // epilogue: lane holds column wrow0 + n, rows (j/4)*8 + half*4 + (j%4) of each 32-row tile
#pragma unroll
    for (int mt = 0; mt < kBM / 32; ++mt)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int r = mt * 32 + (j >> 2) * 8 + half * 4 + (j & 3);
            if (row0 + r < T) {
                float v;
                if constexpr (NMAT == 2) {
                    const float g = acc[0][mt][j];
                    v = g / (1.0f + __expf(-g)) * acc[1][mt][j];
                } else {
                    v = acc[0][mt][j];
                }
                out[(size_t)(out_row0 + r) * ldo + wrow0 + n] = __float2half(v);
            }
        }
}

template <int NMAT>
__device__ __forceinline__ void grouped_gemm_body(const GemmArgs& a) {
    constexpr int kBM = NMAT == 2 ? kBMUp : kBMDown;
    __shared__ __align__(16) __half xt[2 * kBM * kLdsRow];
    __shared__ int arow[kBM];
    const int nseg = a.E + a.n_shared;
    // the shared experts' segments come last in the table and hold the fullest tiles: they go first
    const int ntile = a.tile_start[nseg];
    if ((int)blockIdx.x >= ntile) return;
    const int b = ntile - 1 - (int)blockIdx.x;
    int lo = 0, hi = nseg;                 // last seg with tile_start[seg] <= b
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.tile_start[mid] <= b) lo = mid; else hi = mid;
    }
    const int seg = lo;
    const bool is_shared = seg >= a.E;
    const int local = b - a.tile_start[seg];
    const int nb = is_shared ? a.nb_s : a.nb_r;
    const int mb = local / nb, nblk = local - mb * nb;
    const fate_qexpert* ex = is_shared ? a.shared + (seg - a.E) : a.experts + seg;
    const int sbeg = is_shared ? 0 : a.offsets[seg];
    const int T = is_shared ? a.N : a.offsets[seg + 1] - sbeg;
    const int row0 = mb * kBM;
    const int Nout = a.mode == 0 ? ex->I : a.H;
    const int K = a.mode == 0 ? a.H : ex->I;
    const __half* A = is_shared ? a.A_s : a.A_r;
    const int lda = is_shared ? a.lda_s : a.lda_r;
    if (nblk * kBN >= Nout) return;
    if ((a.mode == 0 ? ex->w1 : ex->w2) == nullptr) {
        if (threadIdx.x == 0) atomicOr(a.status, 1);
        return;
    }
    for (int r = threadIdx.x; r < kBM; r += 256) {
        const int rr = row0 + r < T ? row0 + r : row0;
        int ar;
        if (a.mode == 0) ar = is_shared ? rr : a.perm[sbeg + rr] / a.k;
        else ar = is_shared ? (seg - a.E) * a.N + rr : sbeg + rr;
        arow[r] = ar;
    }
    __syncthreads();
    __half* out = is_shared ? a.out_s : a.out_r;
    const int ldo = is_shared ? a.ldo_s : a.ldo_r;
    const int out_row0 = (is_shared ? (seg - a.E) * a.N : sbeg) + row0;
    // width and group of THIS expert's copy: a layer may hold copies of several widths (the
    // popularity-aware hybrid of section 4.5 moves the least popular experts at 2 bits)
    const int bits = ex->bits, group = ex->group;
    const int kt = bits == 4 ? 64 : (bits == 8 ? 32 : 128);
    if ((bits != 2 && bits != 4 && bits != 8) || group < kt || group % kt || K % group) {
        if (threadIdx.x == 0) atomicOr(a.status, 4);
        return;
    }
    const bool has_z = ex->z1 != nullptr;
    if (has_z && (bits == 8 || ex->z2 == nullptr || ex->z3 == nullptr)) {     // zero-points: 4- and 2-bit formats
        if (threadIdx.x == 0) atomicOr(a.status, 4);
        return;
    }
    if (has_z && bits == 4)
        gemm_tile<4, NMAT, kBM, true>(a, ex, group, row0, T, nblk, arow, xt, out, ldo, out_row0, Nout, K, A, lda);
    else if (has_z)
        gemm_tile<2, NMAT, kBM, true>(a, ex, group, row0, T, nblk, arow, xt, out, ldo, out_row0, Nout, K, A, lda);
    else if (bits == 4)
        gemm_tile<4, NMAT, kBM>(a, ex, group, row0, T, nblk, arow, xt, out, ldo, out_row0, Nout, K, A, lda);
    else if (bits == 2)
        gemm_tile<2, NMAT, kBM>(a, ex, group, row0, T, nblk, arow, xt, out, ldo, out_row0, Nout, K, A, lda);
    else
        gemm_tile<8, NMAT, kBM>(a, ex, group, row0, T, nblk, arow, xt, out, ldo, out_row0, Nout, K, A, lda);
}

// two waves per SIMD for the up GEMM (two matrices: 256 registers), three for the down GEMM
template <int NMAT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void grouped_gemm_kernel(GemmArgs a) {
    grouped_gemm_body<NMAT>(a);
}
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void grouped_gemm_down_kernel(GemmArgs a) {
    grouped_gemm_body<1>(a);
}

// y[t,:] = sum_j w[t,j] * Yp_r[inv_perm[t*k+j], :] + sum_s g_s(t) * Yp_s[s*N+t, :]
__global__ __launch_bounds__(256) void combine_kernel(const __half* __restrict__ yp_r,
                                                      const __half* __restrict__ yp_s,
                                                      const int32_t* __restrict__ inv_perm,
                                                      const float* __restrict__ topk_w,
                                                      const float* __restrict__ sgate, int N, int H, int k,
                                                      int n_shared, float* __restrict__ y32,
                                                      uint16_t* __restrict__ y16) {
    const int t = blockIdx.x;
    for (int c = threadIdx.x; c < (H >> 3); c += 256) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int j = 0; j < k + n_shared; ++j) {
            float wgt;
            const __half* src;
            if (j < k) {
                const int pos = inv_perm[t * k + j];
                if (pos < 0) continue;
                wgt = topk_w[t * k + j];
                src = yp_r + (size_t)pos * H;
            } else {
                wgt = sgate ? sgate[t] : 1.0f;
                src = yp_s + ((size_t)(j - k) * N + t) * H;
            }
            const uint4 v = reinterpret_cast<const uint4*>(src)[c];
            const __half2* h = reinterpret_cast<const __half2*>(&v);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[2 * i] = fmaf(wgt, __low2float(h[i]), acc[2 * i]);
                acc[2 * i + 1] = fmaf(wgt, __high2float(h[i]), acc[2 * i + 1]);
            }
        }
        if (y32) {
            float4* o = reinterpret_cast<float4*>(y32 + (size_t)t * H + c * 8);
            o[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
            o[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
        } else {
            uint32_t o[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                o[i] = f32_to_bf16_bits(acc[2 * i]) | (f32_to_bf16_bits(acc[2 * i + 1]) << 16);
            reinterpret_cast<uint4*>(y16 + (size_t)t * H)[c] = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
}

fate_status launch_ffn_mfma(hipStream_t st, const fate_ffn_desc& d, DecodeArgs da, const MfmaScratch& ms,
                            void* y_out, int phase, const PartSel& sel) {
    if (d.H % kKC || d.I_max % kKC || (d.n_shared && d.I_shared_max % kKC))
        FATE_FAIL(FATE_ESHAPE, "the MFMA path needs H and I to be multiples of %d", kKC);
    const int P = d.N * d.k;
    // the GEMM addresses activation rows with 32-bit element offsets
    const long long amax = std::max({(long long)d.N * d.H, (long long)P * da.ldh_r,
                                     (long long)d.n_shared * d.N * da.ldh_s});
    if (amax >= (1LL << 31))
        FATE_FAIL(FATE_ESHAPE, "the MFMA path needs activation matrices of fewer than 2^31 elements (%lld)", amax);
    const int nseg = d.E + d.n_shared;
    const int nb_r_up = (d.I_max + kBN - 1) / kBN, nb_s_up = d.n_shared ? (d.I_shared_max + kBN - 1) / kBN : 0;
    const int nb_down = (d.H + kBN - 1) / kBN;
    const bool do_up = phase != 2, do_down = phase != 1;
    (void)nseg;
    if (do_up) {
        prefill_prep_kernel<<<sel.first ? d.N : 1, 256, 0, st>>>(da.x, d.N, d.H, d.E, d.n_shared, da.offsets,
                                                                 da.shared_gate, ms.xh, ms.sgate, ms.tab_up, ms.tab_down,
                                                                 nb_r_up, nb_s_up, nb_down, nb_down, sel);
        FATE_HIP(hipGetLastError());
    }
    // upper bounds of the routed row blocks, and the shared experts' row blocks, per GEMM
    const int mb_r_up = P / kBMUp + (d.E < P ? d.E : P), mb_s_up = (d.N + kBMUp - 1) / kBMUp;
    const int mb_r_down = P / kBMDown + (d.E < P ? d.E : P), mb_s_down = (d.N + kBMDown - 1) / kBMDown;
    GemmArgs g{};
    g.experts = da.experts; g.shared = da.shared; g.E = d.E; g.n_shared = d.n_shared; g.N = d.N; g.k = d.k;
    g.offsets = da.offsets; g.perm = da.perm;
    g.bits_r = da.bits_r; g.group_r = da.group_r; g.bits_s = da.bits_s; g.group_s = da.group_s;
    g.status = da.status;
    g.H = d.H;
    if (do_up) {
        g.A_r = ms.xh; g.lda_r = d.H; g.A_s = ms.xh; g.lda_s = d.H; g.mode = 0; g.tile_start = ms.tab_up;
        g.out_r = da.h_r; g.ldo_r = da.ldh_r; g.out_s = da.h_s; g.ldo_s = da.ldh_s;
        g.nb_r = nb_r_up; g.nb_s = nb_s_up;
        const long long grid = (long long)mb_r_up * nb_r_up + (long long)d.n_shared * mb_s_up * nb_s_up;
        if (grid > 0x7fffffffLL) FATE_FAIL(FATE_ESHAPE, "too many tiles");
        grouped_gemm_kernel<2><<<(unsigned)grid, 256, 0, st>>>(g);
        FATE_HIP(hipGetLastError());
    }
    if (do_down) {
        g.A_r = da.h_r; g.lda_r = da.ldh_r; g.A_s = da.h_s; g.lda_s = da.ldh_s; g.mode = 1;
        g.tile_start = ms.tab_down; g.nb_r = nb_down; g.nb_s = nb_down;
        g.out_r = ms.yp_r; g.ldo_r = d.H; g.out_s = ms.yp_s; g.ldo_s = d.H;
        const long long grid = ((long long)mb_r_down + (long long)d.n_shared * mb_s_down) * nb_down;
        if (grid > 0x7fffffffLL) FATE_FAIL(FATE_ESHAPE, "too many tiles");
        grouped_gemm_down_kernel<<<(unsigned)grid, 256, 0, st>>>(g);
        FATE_HIP(hipGetLastError());
        if (sel.last)
            combine_kernel<<<d.N, 256, 0, st>>>(ms.yp_r, ms.yp_s, da.inv_perm, da.topk_w,
                                            da.shared_gate ? ms.sgate : nullptr, d.N, d.H, d.k, d.n_shared,
                                            d.y_is_fp32 ? static_cast<float*>(y_out) : nullptr,
                                            d.y_is_fp32 ? nullptr : static_cast<uint16_t*>(y_out));
        FATE_HIP(hipGetLastError());
    }
    return FATE_OK;
}

}  // namespace fate
