// fate_moe_layer_decode: a whole decode-side MoE layer in two launches (1..8
// tokens): gate logits, softmax / top-k, cross-layer prediction, permutation
// and the quantised expert FFN.
//
// Block ids, in order:
//  routing workgroups: each wave evaluates one gate row (this layer's gate,
//    then the next layer's) for every token and publishes the logit tagged
//    with the call's epoch.  The last one waits for all logits and writes the
//    routing outputs of the API.
//  work blocks: 32 intermediate neurons of one shared expert or of one routed
//    slot.  A routed block polls the tagged logits (the only cross-workgroup
//    dependency on its path), redoes softmax / top-k / permutation for itself
//    in LDS - same code on the same bits as the routing workgroup - and so
//    learns its expert without waiting for another workgroup's bookkeeping.
//    Then: all requests for its W1/W3 row block and W2 column block go out,
//    the waves split the reduction dimension of the up projection, the 32
//    values of h stay in LDS, and each wave multiplies them into its share of
//    the 32-row blocks of W2 and stores weight * partial as a row of its own
//    (device-scope fp32 atomics on y serialise at the memory side and were
//    several times slower than writing the rows out and adding them up).
//  A second, small kernel adds the partial rows into y.
// A workgroup only ever waits for workgroups with lower ids, which the
// dispatcher of its compute die has started before it; every wait is bounded
// and turns into a status bit when it runs out.
// (This header holds the kernel.  layer_decode.hip instantiates the one-item-per-block kernels,
// layer_decode_loop_r*.hip the looping ones, one unit per weight format of the routed experts,
// so that the units build in parallel.)
#pragma once
#include <hip/hip_fp16.h>
#include <algorithm>
#include "common.h"
#include "qformat.h"
#include "decode_device.h"
#include "route_device.h"
#include "layer_decode.h"
#include "layer_decode_lds.h"

namespace fate {

constexpr int kSpinMax = 1 << 18;
constexpr int kUpRing = 8;        // tiles in flight per matrix per wave
constexpr int kDownRing = 8;      // W2 pieces in flight per wave

struct TaggedStore {
    unsigned long long* zq; int N, E; uint32_t tag;
    __device__ __forceinline__ void operator()(int g, int t, int e, float v) const {
        __hip_atomic_store(zq + ((size_t)g * N + t) * E + e,
                           ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(v),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
};
struct LdsLoad {
    const float* zl; int N, E;
    __device__ __forceinline__ float operator()(int g, int t, int e) const { return zl[((size_t)g * N + t) * E + e]; }
};

// Every thread of the workgroup calls it: polls n tagged logits until all
// carry this call's tag and leaves their values in dst (LDS).
__device__ __forceinline__ bool wait_logits(const unsigned long long* zq, int n, uint32_t tag, float* dst) {
    for (int it = 0; it < kSpinMax; ++it) {
        int ok = 1;
        for (int i = threadIdx.x; i < n; i += kLayerThreads) {
            const unsigned long long v = ld_dev(zq + i);
            if ((uint32_t)(v >> 32) == tag) dst[i] = __uint_as_float((uint32_t)v);
            else ok = 0;
        }
        if (__syncthreads_and(ok)) return true;
        __builtin_amdgcn_s_sleep(8);
    }
    return false;
}

__device__ __forceinline__ void route_role(const LayerArgs& a, int b, uint32_t tag, char* dyn, FusedRouteSmem& rsm) {
    const int tid = threadIdx.x;
    const FusedRouteArgs& r = a.r;
    fused_gate_rows(r, b, TaggedStore{a.zq, r.N, r.E, tag});
    if (b != a.nb_route - 1) return;
    // the routing outputs of the API (consumers inside this launch do not read them)
    float* zl = reinterpret_cast<float*>(dyn);
    const int n = (r.Wg2 ? 2 : 1) * r.N * r.E;
    if (!wait_logits(a.zq, n, tag, zl)) {
        if (tid == 0) atomicOr(a.status, 2);
        return;
    }
    fused_select(r, rsm, nullptr, LdsLoad{zl, r.N, r.E});
}

// ---- Fast body: shapes whose per-wave share is a whole number of register rings ----
//
// The codes enter the matrix cores as u + C (C = 1024 or 64 for int4 depending on the nibble's
// position, 1024 for int8: one v_and_or_b32 / v_perm_b32 per pair of codes and nothing else),
// and the constant part leaves afterwards:  sum_k x_k q_k = sum_k x_k (u_k + C_k) - sum_k x_k (C_k + zero).
// The second sum does not depend on the weight row, so it is taken once per token and group
// from the fp16 activations in LDS.  u + C and x are exact in fp16, their products exact in
// fp32; the fp32 accumulation carries terms about (C + zero) / |q| times larger than the
// result, which costs that factor times 2^-24 in relative accuracy per addition.
struct BiasConst {
    uint32_t m0, b0, m1, b1;    // int4: masks / exponent bits of the two nibble positions
};
__device__ __forceinline__ BiasConst bias_const() {
    return BiasConst{vgpr_const(0x000f000fu), vgpr_const(0x64006400u), vgpr_const(0x00f000f0u), vgpr_const(0x54005400u)};
}
// one dword of eight int4 codes -> 8 fp16 values u + C in column order (C = 1024, 1024, 64, 64, 1024, 1024, 64, 64)
__device__ __forceinline__ f16x8_t biased_int4(uint32_t r, const BiasConst& c) {
    const uint32_t hi = r >> 8;
    const uint32_t w0 = (r & c.m0) | c.b0, w1 = (r & c.m1) | c.b1, w2 = (hi & c.m0) | c.b0, w3 = (hi & c.m1) | c.b1;
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
    return __builtin_bit_cast(f16x8_t, u32x4_t{w0, w1, w2, w3});
}
// two dwords of four int8 codes each -> 8 fp16 values 1024 + u
__device__ __forceinline__ f16x8_t biased_int8(uint32_t r0, uint32_t r1) {
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
    return __builtin_bit_cast(f16x8_t, u32x4_t{__builtin_amdgcn_perm(0x64646464u, r0, 0x04010400u),
                                               __builtin_amdgcn_perm(0x64646464u, r0, 0x04030402u),
                                               __builtin_amdgcn_perm(0x64646464u, r1, 0x04010400u),
                                               __builtin_amdgcn_perm(0x64646464u, r1, 0x04030402u)});
}
template <int BITS>
__device__ __forceinline__ void biased_tile(const uint4& raw, const BiasConst& c, f16x8_t* b) {
    if constexpr (BITS == 4) {
        b[0] = biased_int4(raw.x, c); b[1] = biased_int4(raw.y, c);
        b[2] = biased_int4(raw.z, c); b[3] = biased_int4(raw.w, c);
    } else {
        b[0] = biased_int8(raw.x, raw.y); b[1] = biased_int8(raw.z, raw.w);
    }
}
// sum_k v_k (C_k + zero) over 8 fp16 values in column order
template <int BITS>
__device__ __forceinline__ float bias_dot8(const uint4& v, float acc) {
    const f16x2_t cA = BITS == 4 ? f16x2_t{(_Float16)1032.f, (_Float16)1032.f} : f16x2_t{(_Float16)1152.f, (_Float16)1152.f};
    const f16x2_t cB = BITS == 4 ? f16x2_t{(_Float16)72.f, (_Float16)72.f} : cA;
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, v.x), cA, acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, v.y), cB, acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, v.z), cA, acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, v.w), cB, acc, false);
    return acc;
}
__device__ __forceinline__ float bias_of_column(int bits, int col) {
    return bits == 4 ? ((col & 2) ? 72.f : 1032.f) : 1152.f;
}

struct WorkCtx {
    int tid;
    int N, H, I, T, kb, wb, ntp, ldx;
    bool is_shared, defer_x;
    fate_qexpert ex;
    _Float16 *xs, *hs;
    float *red, *wtok, *cx, *ch;
    const int32_t *tokid, *pairq;
    float* part;
    size_t part_stride;
};

constexpr int kCxLd = kTokPass + 1;      // bias sums per group: tokens 0..7 and a zero for absent rows

// one ring of the up projection: D tiles of both matrices, straight-line so that the compiler
// can wait for exactly the tile it needs
// (mid: called once half of the ring's registers are free again)
template <int BITS, int TPG, bool REFILL, class Mid>
__device__ __forceinline__ void up_round(uint4 (&raw)[2][kUpRing], uint32_t (&scr)[2][kUpRing / TPG], const gu4_t* wt,
                                         const gu16_t* sc, int srows, int round, const _Float16* xa, const float* cxg,
                                         const int (&ctok)[4], const BiasConst& bc, float (&out)[2][4], Mid&& mid) {
    constexpr int KT = QFmt<BITS>::KT, S = QFmt<BITS>::MSTEPS, D = kUpRing, GR = D / TPG;
    static_assert(GR >= 2, "mid() runs between two groups of a ring");
    const f32x16_t zero = f32x16_zero();
#pragma unroll
    for (int jg = 0; jg < GR; ++jg) {
        float s[2], cj[4];
        f32x16_t acc[2];
        if (jg == (GR + 1) / 2) mid();
#pragma unroll
        for (int i = 0; i < 2; ++i) s[i] = half_bits_to_float(scr[i][jg]);
        if constexpr (REFILL) {
#pragma unroll
            for (int i = 0; i < 2; ++i) scr[i][jg] = sc[i][(size_t)((round + 1) * GR + jg) * srows];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) cj[j] = cxg[(round * GR + jg) * kCxLd + ctok[j]];
#pragma unroll
        for (int tl = 0; tl < TPG; ++tl) {
            const int j = jg * TPG + tl;
            const _Float16* xt = xa + (round * D + j) * KT;
            f16x8_t av[S];
#pragma unroll
            for (int st = 0; st < S; ++st) av[st] = *reinterpret_cast<const f16x8_t*>(xt + 8 * st);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                f16x8_t b[S];
                biased_tile<BITS>(raw[i][j], bc, b);
                if constexpr (REFILL) raw[i][j] = wt[i][(size_t)((round + 1) * D + j) * 64];
#pragma unroll
                for (int st = 0; st < S; ++st)
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[st], b[st], (tl == 0 && st == 0) ? zero : acc[i],
                                                                    0, 0, 0);
            }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) out[i][j] = fmaf(s[i], acc[i][j] - cj[j], out[i][j]);
    }
}

template <int BITS>
struct DownPiece;
template <>
struct DownPiece<4> { typedef uint2 type; static constexpr int NQ = 16; };
template <>
struct DownPiece<8> { typedef uint4 type; static constexpr int NQ = 8; };

template <int BITS, int TPG, class LoadX, class StoreX, class Gate>
__device__ __forceinline__ void body_fast(const WorkCtx& c, LoadX&& load_x, StoreX&& store_x, Gate&& shared_gate) {
    constexpr int KT = QFmt<BITS>::KT, D = kUpRing, GR = D / TPG, NQ = DownPiece<BITS>::NQ;
    typedef typename DownPiece<BITS>::type piece_t;
    typedef const FATE_GLOBAL piece_t* gpiece_t;
    const int tid = c.tid, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, half = lane >> 5;
    const int H = c.H, I = c.I, T = c.T, N = c.N, kb = c.kb;
    const int tiles_k = H / KT;
    const int tw = tiles_k / kLayerWaves;            // tiles per wave and matrix, a multiple of D
    const int rounds = tw / D;
    const int g_beg = wave * (tw / TPG);
    const gu4_t wt[2] = {as_global<uint4>(c.ex.w1) + ((size_t)kb * tiles_k + wave * tw) * 64 + lane,
                         as_global<uint4>(c.ex.w3) + ((size_t)kb * tiles_k + wave * tw) * 64 + lane};
    const gu16_t sc[2] = {as_global<uint16_t>(c.ex.s1) + (size_t)g_beg * I + kb * 32 + n,
                          as_global<uint16_t>(c.ex.s3) + (size_t)g_beg * I + kb * 32 + n};
    // W2: the 32 columns of this block in every 32-row block; a wave takes every kLayerWaves-th
    // row block, starting from a block-dependent one.  int4: the 32 codes of a row are the 16
    // bytes of one lane of the tile; the two half-waves fetch 8 of them each (columns 0..15 and
    // 16..31 of the block), so every lane feeds the matrix core.  int8: one whole tile.
    const int tiles_k2 = I / KT;
    const int nq = (H >> 5) / kLayerWaves;           // row blocks per wave, a multiple of NQ
    const int qrot = c.wb % nq;
    const char FATE_GLOBAL* w2b = as_global<char>(c.ex.w2) +
        (BITS == 4 ? ((size_t)(kb >> 1) * 1024 + ((kb & 1) * 32 + n) * 16 + 8 * half) : ((size_t)kb * 1024 + lane * 16));
    const gu16_t s2 = as_global<uint16_t>(c.ex.s2) + (size_t)(kb * kLayerNeurons / (KT * TPG)) * H + n;
    auto rb_of = [&](int q) { int qq = q + qrot; if (qq >= nq) qq -= nq; return wave + kLayerWaves * qq; };

    if (c.defer_x) load_x();
    uint4 raw[2][D];
    uint32_t scr[2][GR];
#pragma unroll
    for (int j = 0; j < D; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i) raw[i][j] = wt[i][(size_t)j * 64];
#pragma unroll
    for (int jg = 0; jg < GR; ++jg)
#pragma unroll
        for (int i = 0; i < 2; ++i) scr[i][jg] = sc[i][(size_t)jg * I];
    piece_t dA[NQ], dB[NQ];
    uint32_t sA[NQ], sB[NQ];
    auto issue_w = [&](piece_t (&d)[NQ], int chunk) {
#pragma unroll
        for (int u = 0; u < NQ; ++u)
            d[u] = *reinterpret_cast<gpiece_t>(w2b + (size_t)rb_of(chunk * NQ + u) * tiles_k2 * 1024);
    };
    auto issue_s = [&](uint32_t (&sd)[NQ], int chunk) {
#pragma unroll
        for (int u = 0; u < NQ; ++u) sd[u] = s2[rb_of(chunk * NQ + u) * 32];
    };
    auto issue = [&](piece_t (&d)[NQ], uint32_t (&sd)[NQ], int chunk) { issue_w(d, chunk); issue_s(sd, chunk); };
    issue_w(dA, 0);           // its scales follow once half of the ring has been consumed
    if (c.defer_x) store_x(true);
    if (c.is_shared) shared_gate();
    lds_barrier();            // x, token ids and weights are in LDS
    // bias sums of x for this wave's groups: 8 lanes per token, each a slice of the group
    {
        constexpr int per = KT * TPG / 8;            // columns per lane
        const int t = lane >> 3, sub = lane & 7;
        const _Float16* xp = c.xs + (t < N ? t : N) * c.ldx + (size_t)g_beg * (KT * TPG) + sub * per;
        for (int g = 0; g < tw / TPG; ++g) {
            float sum = 0.f;
#pragma unroll
            for (int v = 0; v < per / 8; ++v)
                sum = bias_dot8<BITS>(*reinterpret_cast<const uint4*>(xp + (size_t)g * (KT * TPG) + 8 * v), sum);
            sum += __shfl_xor(sum, 1, 64);
            sum += __shfl_xor(sum, 2, 64);
            sum += __shfl_xor(sum, 4, 64);
            if (sub == 0) c.cx[(g_beg + g) * kCxLd + t] = sum;
            if (lane == 1) c.cx[(g_beg + g) * kCxLd + kTokPass] = 0.f;
        }
    }
    const BiasConst bc = bias_const();
    float out[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    const int arow = n < T ? c.tokid[n] : N;
    int ctok[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) ctok[j] = 4 * half + j < T ? c.tokid[4 * half + j] : kTokPass;
    const _Float16* xa = c.xs + arow * c.ldx + half * (KT / 2) + (size_t)wave * tw * KT;
    const float* cxg = c.cx + g_beg * kCxLd;
    for (int r = 0; r + 1 < rounds; ++r)
        up_round<BITS, TPG, true>(raw, scr, wt, sc, I, r, xa, cxg, ctok, bc, out, [] {});
    up_round<BITS, TPG, false>(raw, scr, wt, sc, I, rounds - 1, xa, cxg, ctok, bc, out, [&] { issue_s(sA, 0); });
    const int nchunk = nq / NQ;
    if (nchunk > 1) issue(dB, sB, 1);     // the ring's registers are free now
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (4 * half + j < c.ntp) c.red[((wave * 2 + i) * c.ntp + 4 * half + j) * 32 + n] = out[i][j];
    lds_barrier();
    if (tid < T * kLayerNeurons) {        // T <= 8 rows of 32: one value per thread, one row per half-wave
        const int t = tid >> 5;
        float a1 = 0.f, a3 = 0.f;
#pragma unroll
        for (int w = 0; w < kLayerWaves; ++w) {
            a1 += c.red[((w * 2) * c.ntp + t) * 32 + n];
            a3 += c.red[((w * 2 + 1) * c.ntp + t) * 32 + n];
        }
        const _Float16 hv = (_Float16)(a1 / (1.0f + expf(-a1)) * a3);
        c.hs[t * kHsLd + n] = hv;
        float bsum = (float)hv * bias_of_column(BITS, n);
        bsum += __shfl_xor(bsum, 1, 64);
        bsum += __shfl_xor(bsum, 2, 64);
        bsum += __shfl_xor(bsum, 4, 64);
        bsum += __shfl_xor(bsum, 8, 64);
        bsum += __shfl_xor(bsum, 16, 64);
        if (n == 0) c.ch[t] = bsum;
    }
    lds_barrier();
    // down projection: two matrix-core steps per piece (16 columns of h per half-wave)
    const _Float16* ha = c.hs + (n < T ? n : kTokPass) * kHsLd + 16 * half;
    float wj[4], chj[4];
    float* rowj[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int t = 4 * half + j;
        wj[j] = t < T ? c.wtok[t] : 0.f;
        chj[j] = t < T ? c.ch[t] : 0.f;
        rowj[j] = c.part + (size_t)(t < T ? (c.is_shared ? t : c.pairq[t]) : 0) * c.part_stride + n;
    }
    const f16x8_t av0 = *reinterpret_cast<const f16x8_t*>(ha), av1 = *reinterpret_cast<const f16x8_t*>(ha + 8);
    const f32x16_t zero = f32x16_zero();
    // four pieces at a time, each with its own accumulator: the two dependent matrix-core
    // steps of one piece overlap with those of the others
    auto process = [&](piece_t (&d)[NQ], uint32_t (&sd)[NQ], int chunk) {
#pragma unroll
        for (int u0 = 0; u0 < NQ; u0 += 4) {
            f32x16_t acc[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                f16x8_t b0;
                if constexpr (BITS == 4) b0 = biased_int4(d[u0 + v].x, bc);
                else b0 = biased_int8(d[u0 + v].x, d[u0 + v].y);
                acc[v] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av0, b0, zero, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                f16x8_t b1;
                if constexpr (BITS == 4) b1 = biased_int4(d[u0 + v].y, bc);
                else b1 = biased_int8(d[u0 + v].z, d[u0 + v].w);
                acc[v] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av1, b1, acc[v], 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int rb = rb_of(chunk * NQ + u0 + v);
                const float s = half_bits_to_float(sd[u0 + v]);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (4 * half + j < T) rowj[j][rb * 32] = (wj[j] * s) * (acc[v][j] - chj[j]);
            }
        }
    };
    for (int ch = 0; ch < nchunk; ch += 2) {
        process(dA, sA, ch);
        if (ch + 2 < nchunk) issue(dA, sA, ch + 2);
        if (ch + 1 < nchunk) {
            process(dB, sB, ch + 1);
            if (ch + 3 < nchunk) issue(dB, sB, ch + 3);
        }
    }
}


// BR/TR: bits and tiles per group of the routed experts, BS/TS: of the shared experts (equal to
// the routed ones when the layer has none).  One kernel per combination keeps the code a
// workgroup runs through small: instruction fetch at the cold start of a launch is on the
// critical path of the first weight requests.
//
// One work item (wb) of a work block; with LOOP a block runs several in turn (launches with more
// items than workgroups that fit on the device) and state, kept by the caller across the items
// of a block, says what is already in LDS: bit 0 = x and the zero rows, bit 1 = the routing of
// all tokens; bit 2 = a wait ran out, stop.  Without LOOP state is not used.
template <int BR, int TR, int BS, int TS, bool LOOP>
__device__ __forceinline__ void work_role(const LayerArgs& a, int wb, uint32_t tag, char* dyn, int& state) {
    int tid0 = threadIdx.x;
    // (looping kernels: the thread index is made opaque per item, so that what is derived from it
    // is recomputed instead of being kept in registers across the whole body of every item)
    if constexpr (LOOP) asm volatile("" : "+v"(tid0));
    const int tid = tid0, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, half = lane >> 5;
    const int N = a.r.N, H = a.r.H, E = a.r.E, k = a.r.k;
    const WorkLds L = work_lds(N, H, E, k);
    _Float16* xs = reinterpret_cast<_Float16*>(dyn + L.xs);
    _Float16* hs = reinterpret_cast<_Float16*>(dyn + L.hs);
    float* red = reinterpret_cast<float*>(dyn + L.red);
    int32_t* tokid = reinterpret_cast<int32_t*>(dyn + L.tokid);
    float* wtok = reinterpret_cast<float*>(dyn + L.wtok);
    const int ldx = H + kLdsPad, nvec = H >> 3;
    const int ntp = N < kTokPass ? N : kTokPass;
    const int nsh = a.n_shared * a.nkb_s;
    const bool is_shared = wb < nsh;

    // Activations of every token go to LDS as fp16 (the routing result only picks rows later),
    // plus zero rows.  A routed block does this while it has nothing else to do; a shared block
    // with little x requests it first, then its weights, and stores x once it has arrived.
    const bool x_one = N * nvec <= kLayerThreads;      // one 16-byte piece per thread covers x
    uint4 xv = make_uint4(0, 0, 0, 0);
    auto load_x = [&]() {
        if (tid < N * nvec) xv = reinterpret_cast<const uint4*>(a.r.x)[tid];
    };
    auto store_x = [&](bool from_reg) {
        if (from_reg) {
            if (tid < N * nvec) {
                const int t = tid / nvec, c = tid - t * nvec;
                *reinterpret_cast<uint4*>(xs + t * ldx + c * 8) = bf16x8_to_f16x8(xv);
            }
        } else {
            const uint4* xg = reinterpret_cast<const uint4*>(a.r.x);
            for (int idx = tid; idx < N * nvec; idx += kLayerThreads) {
                const int t = idx / nvec, c = idx - t * nvec;
                *reinterpret_cast<uint4*>(xs + t * ldx + c * 8) = bf16x8_to_f16x8(xg[idx]);
            }
        }
        for (int c = tid; c < (ldx >> 3); c += kLayerThreads)
            *reinterpret_cast<uint4*>(xs + N * ldx + c * 8) = make_uint4(0, 0, 0, 0);
        for (int c = tid; c < (kHsLd >> 3); c += kLayerThreads)
            *reinterpret_cast<uint4*>(hs + kTokPass * kHsLd + c * 8) = make_uint4(0, 0, 0, 0);
    };
    const bool x_ready = LOOP && (state & 1);
    const bool defer_x = is_shared && x_one && !x_ready;
    if (!defer_x && !x_ready) store_x(false);
    if constexpr (LOOP) state |= 1;

    fate_qexpert ex;
    int kb, T, bits, group;
    int32_t* pairq = reinterpret_cast<int32_t*>(dyn + L.pairq);  // routed: original pair index of each of the T rows
    float* part;                  // where this block's weighted partial output rows go
    size_t part_stride;           // floats between the rows of consecutive tokens of this block
    if (is_shared) {
        const int s = wb / a.nkb_s;
        kb = wb - s * a.nkb_s;
        ex = a.shared[s];
        T = N;
        bits = a.bits_s; group = a.group_s;
        part = a.part_s + ((size_t)s * a.nkb_s + kb) * N * H;
        part_stride = H;
        if (tid < N) tokid[tid] = tid;
    } else {
        uint4* tab = reinterpret_cast<uint4*>(dyn + L.tab);
        float* zl = reinterpret_cast<float*>(dyn + L.zl);
        int32_t* ids = reinterpret_cast<int32_t*>(dyn + L.ids);
        float* wv = reinterpret_cast<float*>(dyn + L.w);
        if (!LOOP || !(state & 2)) {
            // the expert table travels while the logits are awaited
            const uint4* src = reinterpret_cast<const uint4*>(a.experts);
            for (int i = tid; i < E * (int)(sizeof(fate_qexpert) / 16); i += kLayerThreads) tab[i] = src[i];
            if (!wait_logits(a.zq, N * E, tag, zl)) {
                if (tid == 0) atomicOr(a.status, 2);
                if constexpr (LOOP) state |= 4;
                return;
            }
            for (int t = wave; t < N; t += kLayerWaves)
                wave_softmax_topk_rounds(zl + t * E, E, k, a.r.renorm, ids + t * k, wv + t * k);
            __syncthreads();
            if constexpr (LOOP) {
                // every slot's expert and rows, once per block: the items only look them up
                int32_t* slots = reinterpret_cast<int32_t*>(dyn + L.slots);
                for (int i = tid; i < kLayerMaxP; i += kLayerThreads) slots[i * kSlotWords] = -1;
                __syncthreads();
                if (wave == 0) wave_slot_table(ids, wv, N * k, E, k, 0u, kTokPass, slots);
                __syncthreads();
                state |= 2;
            }
        }
        const int rwb = wb - nsh;
        const int slot = rwb / a.nkb_r;
        kb = rwb - slot * a.nkb_r;
        if constexpr (LOOP) {
            int32_t* st = reinterpret_cast<int32_t*>(dyn + L.slots) + slot * kSlotWords;
            const int e = st[0];
            if (e < 0) return;                // fewer activated experts than slots: no pair, nothing to write
            T = st[1];
            tokid = st + 2;                   // this item's rows live in the slot's entry
            pairq = st + 2 + kTokPass;
            wtok = reinterpret_cast<float*>(st + 2 + 2 * kTokPass);
            ex = reinterpret_cast<const fate_qexpert*>(tab)[e];
            bits = a.bits_r; group = a.group_r;
        } else {
            int pos;
            const int e = wave_slot_expert(ids, N * k, E, slot, &T, &pos);     // same in every wave
            if (e < 0) return;                    // fewer activated experts than slots: no pair, nothing to write
            ex = reinterpret_cast<const fate_qexpert*>(tab)[e];
            bits = a.bits_r; group = a.group_r;
            if (wave == 0 && pos >= 0) {
                tokid[pos] = lane / k;
                wtok[pos] = wv[lane];
                pairq[pos] = lane;
            }
        }
        part = a.part_r + (size_t)kb * H;
        part_stride = (size_t)a.nkb_r * H;    // row of pair q: part + q * part_stride
    }
    const int I = ex.I;
    // (an entry of another width than the call's - a low-width copy left by a prefill - counts as absent)
    const bool absent = ex.w1 == nullptr || ex.w3 == nullptr || ex.w2 == nullptr || ex.bits != bits ||
                        ex.group != group || ex.z1 != nullptr;
    if (kb * kLayerNeurons >= I || absent) {
        // nothing to compute, but the reduction reads this block's rows: they must be zero
        if (absent && tid == 0) atomicOr(a.status, 1);
        if (LOOP && defer_x) store_x(false);  // a later item of this block expects x in LDS
        __syncthreads();
        for (int idx = tid; idx < T * (H >> 2); idx += kLayerThreads) {
            const int t = idx / (H >> 2), c = idx - t * (H >> 2);
            float* row = part + (size_t)(is_shared ? t : pairq[t]) * part_stride;
            *reinterpret_cast<float4*>(row + 4 * c) = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        return;
    }
    const int KT = bits == 4 ? 64 : 32;
    const int tpg = group / KT;
    const int G = H / group;                 // groups along the reduction dimension of W1 / W3
    const int tiles_k = H / KT;
    const int g_beg = G * wave / kLayerWaves, g_end = G * (wave + 1) / kLayerWaves;
    gu4_t wt[2] = {as_global<uint4>(ex.w1) + (size_t)kb * tiles_k * 64 + lane,
                   as_global<uint4>(ex.w3) + (size_t)kb * tiles_k * 64 + lane};
    gu16_t sc[2] = {as_global<uint16_t>(ex.s1) + kb * 32 + n, as_global<uint16_t>(ex.s3) + kb * 32 + n};
    // W2: the 32 columns [kb*32, kb*32+32) of every 32-row block.  int8: one whole tile per row
    // block; int4: the half of a 64-column tile that the lanes of one half-wave own (the other
    // lanes load nothing and their activation operand is zero).  This wave takes every
    // kLayerWaves-th row block, starting from a block-dependent one.
    const int tiles_k2 = I / KT;
    const int g2 = kb * kLayerNeurons / group;
    const int nrb = H >> 5;
    const int nq = (nrb - wave + kLayerWaves - 1) / kLayerWaves;     // row blocks of this wave
    const int qrot = nq > 0 ? wb % nq : 0;
    const int kt2 = bits == 4 ? (kb >> 1) : kb;
    const bool mine = bits == 4 ? (half == (kb & 1)) : true;
    gu4_t w2 = as_global<uint4>(ex.w2) + (size_t)kt2 * 64 + lane;
    gu16_t s2 = as_global<uint16_t>(ex.s2) + (size_t)g2 * H + n;
    auto rb_of = [&](int q) { int qq = q + qrot; if (qq >= nq) qq -= nq; return wave + kLayerWaves * qq; };
    // sigmoid gate of a shared expert (after the weight requests have gone out)
    auto shared_gate = [&]() {
        if (a.shared_gate != nullptr) {
            for (int t = wave; t < N; t += kLayerWaves) {
                const float g = wave_sigmoid_dot_bf16(reinterpret_cast<const uint4*>(a.r.x) + (size_t)t * nvec,
                                                      reinterpret_cast<const uint4*>(a.shared_gate), nvec);
                if (lane == 0) wtok[t] = g;
            }
        } else if (tid < N) {
            wtok[tid] = 1.0f;
        }
    };

#define FATE_LAYER_BODY(BITS, TPG)                                                                        \
    {                                                                                                     \
        constexpr int S = QFmt<BITS>::MSTEPS;                                                             \
        if (defer_x) load_x();                                                                            \
        TileRing<2, kUpRing, TPG> ring;                                                                   \
        ring_start<2, kUpRing, TPG>(ring, wt, sc, I, g_beg, g_end);                                          \
        /* W2 pieces behind them: two register sets of kDownRing pieces, filled in turn */             \
        uint4 dA[kDownRing], dB[kDownRing];                                                               \
        uint32_t sA[kDownRing], sB[kDownRing];                                                            \
        auto issue = [&](uint4 (&d)[kDownRing], uint32_t (&sd)[kDownRing], int chunk) {                   \
            _Pragma("unroll")                                                                             \
            for (int u = 0; u < kDownRing; ++u) {                                                         \
                const int q = chunk * kDownRing + u;                                                      \
                d[u] = make_uint4(0, 0, 0, 0);                                                            \
                if (q < nq) {                                                                             \
                    const int rb = rb_of(q);                                                              \
                    if (mine) d[u] = w2[(size_t)rb * tiles_k2 * 64];                                      \
                    sd[u] = s2[rb * 32];                                                                  \
                }                                                                                         \
            }                                                                                             \
        };                                                                                                \
        issue(dA, sA, 0);                                                                                 \
        if (defer_x) store_x(true);                                                                       \
        if (is_shared) shared_gate();                                                                     \
        lds_barrier();            /* x, token ids and weights are in LDS */                               \
        float out[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};                                   \
        const int arow = n < T ? tokid[n] : N;                                                            \
        ring_run<BITS, TPG, 2, kUpRing>(ring, wt, sc, I, g_beg, g_end,                                      \
                                        xs + arow * ldx + half * (QFmt<BITS>::KT / 2), 0, out);           \
        issue(dB, sB, 1);         /* the ring's registers are free now */                                 \
        _Pragma("unroll")                                                                                 \
        for (int i = 0; i < 2; ++i)                                                                       \
            _Pragma("unroll")                                                                             \
            for (int j = 0; j < 4; ++j)                                                                   \
                if (4 * half + j < ntp) red[((wave * 2 + i) * ntp + 4 * half + j) * 32 + n] = out[i][j];  \
        lds_barrier();                                                                                    \
        for (int idx = tid; idx < T * kLayerNeurons; idx += kLayerThreads) {                              \
            const int t = idx >> 5, n32 = idx & 31;                                                       \
            float a1 = 0.f, a3 = 0.f;                                                                     \
            _Pragma("unroll")                                                                             \
            for (int w = 0; w < kLayerWaves; ++w) {                                                       \
                a1 += red[((w * 2) * ntp + t) * 32 + n32];                                                \
                a3 += red[((w * 2 + 1) * ntp + t) * 32 + n32];                                            \
            }                                                                                             \
            hs[t * kHsLd + n32] = (_Float16)(a1 / (1.0f + expf(-a1)) * a3);                               \
        }                                                                                                 \
        lds_barrier();                                                                                    \
        /* down projection of the 32 values of h: int8 spreads them over both half-waves (16 each),  */  \
        /* int4 keeps them in the half-wave that owns the columns                                    */  \
        const bool arow_ok = n < T && mine;                                                               \
        const _Float16* ha = hs + (arow_ok ? n : kTokPass) * kHsLd + (BITS == 8 ? half * 16 : 0);         \
        float wj[4];                                                                                      \
        float* rowj[4];                                                                                   \
        _Pragma("unroll")                                                                                 \
        for (int j = 0; j < 4; ++j) {                                                                     \
            const int t = 4 * half + j;                                                                   \
            wj[j] = t < T ? wtok[t] : 0.f;                                                                \
            rowj[j] = part + (size_t)(t < T ? (is_shared ? t : pairq[t]) : 0) * part_stride + n;          \
        }                                                                                                 \
        f16x8_t av[S];                                                                                    \
        _Pragma("unroll")                                                                                 \
        for (int st = 0; st < S; ++st) av[st] = *reinterpret_cast<const f16x8_t*>(ha + 8 * st);           \
        const f32x16_t zero = f32x16_zero();                                                              \
        auto process = [&](uint4 (&d)[kDownRing], uint32_t (&sd)[kDownRing], int chunk) {                 \
            _Pragma("unroll")                                                                             \
            for (int u = 0; u < kDownRing; ++u) {                                                         \
                const int q = chunk * kDownRing + u;                                                      \
                if (q < nq) {                                                                             \
                    const int rb = rb_of(q);                                                              \
                    const float s = half_bits_to_float(sd[u]);                                            \
                    f16x8_t bq[S];                                                                        \
                    codes_to_f16<BITS>(d[u], bq);                                                         \
                    f32x16_t acc;                                                                         \
                    _Pragma("unroll")                                                                     \
                    for (int st = 0; st < S; ++st)                                                        \
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[st], bq[st], st == 0 ? zero : acc, \
                                                                     0, 0, 0);                            \
                    _Pragma("unroll")                                                                     \
                    for (int j = 0; j < 4; ++j)                                                           \
                        if (4 * half + j < T) rowj[j][rb * 32] = wj[j] * (s * acc[j]);                    \
                }                                                                                         \
            }                                                                                             \
        };                                                                                                \
        const int nchunk = (nq + kDownRing - 1) / kDownRing;                                              \
        for (int c = 0; c < nchunk; c += 2) {                                                             \
            process(dA, sA, c);                                                                           \
            if (c + 2 < nchunk) issue(dA, sA, c + 2);                                                     \
            if (c + 1 < nchunk) {                                                                         \
                process(dB, sB, c + 1);                                                                   \
                if (c + 3 < nchunk) issue(dB, sB, c + 3);                                                 \
            }                                                                                             \
        }                                                                                                 \
    }
    // a whole number of rings per wave: the straight-line body
    const bool fast = H % (kLayerWaves * kUpRing * KT) == 0 && I % KT == 0;
    WorkCtx cx;
    cx.tid = tid;
    cx.N = N; cx.H = H; cx.I = I; cx.T = T; cx.kb = kb; cx.wb = wb; cx.ntp = ntp; cx.ldx = ldx;
    cx.is_shared = is_shared; cx.defer_x = defer_x; cx.ex = ex; cx.xs = xs; cx.hs = hs; cx.red = red; cx.wtok = wtok;
    cx.cx = reinterpret_cast<float*>(dyn + L.cx); cx.ch = reinterpret_cast<float*>(dyn + L.ch);
    cx.tokid = tokid; cx.pairq = pairq; cx.part = part; cx.part_stride = part_stride;
#define FATE_LAYER_FAST(BITS, TPG) body_fast<BITS, TPG>(cx, load_x, store_x, shared_gate);
    if constexpr (BR == BS && TR == TS) {
        if (fast) { FATE_LAYER_FAST(BR, TR) }
        else { FATE_LAYER_BODY(BR, TR) }
    } else {
        if (is_shared) {
            if (fast) { FATE_LAYER_FAST(BS, TS) }
            else { FATE_LAYER_BODY(BS, TS) }
        } else {
            if (fast) { FATE_LAYER_FAST(BR, TR) }
            else { FATE_LAYER_BODY(BR, TR) }
        }
    }
#undef FATE_LAYER_FAST
#undef FATE_LAYER_BODY
}

// LOOP: a work block takes every nwork-th item instead of exactly one (launches with more items
// than the device holds workgroups: the routing of all tokens, x and the expert table are then
// set up once per block, not once per item).  The loop keeps more values alive and spills a few
// registers, so launches that fit use the kernel without it.
template <int BR, int TR, int BS, int TS, bool LOOP>
__global__ __launch_bounds__(kLayerThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void moe_layer_decode_kernel(LayerArgs a) {
    extern __shared__ uint4 smem[];
    __shared__ FusedRouteSmem rsm;
    char* dyn = reinterpret_cast<char*>(smem);
    uint32_t tag = (uint32_t)ld_dev(a.sync) + 1u;
    if (tag == 0u) tag = 1u;         // a zero-filled workspace must never look current
    const int b = blockIdx.x;
    if (b < a.nb_route) {
        route_role(a, b, tag, dyn, rsm);
    } else {
        int state = 0;
        if constexpr (LOOP) {
            for (int item = b - a.nb_route; item < a.nitems; item += a.nwork) {
                if (state) lds_barrier();     // every wave is done with the previous item's LDS
                work_role<BR, TR, BS, TS, true>(a, item, tag, dyn, state);
                if (state & 4) break;
            }
        } else {
            work_role<BR, TR, BS, TS, false>(a, b - a.nb_route, tag, dyn, state);
        }
    }
    // the workgroup that leaves last opens the next epoch
    __syncthreads();
    if (threadIdx.x == 0 && atomicAdd(a.sync + 1, 1) == (int)gridDim.x - 1) {
        st_dev(a.sync + 1, 0);
        st_dev(a.sync, (int32_t)tag);
    }
}

template <int BR, int TR, int BS, int TS, bool LOOP>
static fate_status launch_layer_kernel_v(hipStream_t st, int grid, int lds_bytes, int lds_max, const LayerArgs& a) {
    static bool attr_done = false;
    if (!attr_done) {
        FATE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(moe_layer_decode_kernel<BR, TR, BS, TS, LOOP>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds_max));
        attr_done = true;
    }
    moe_layer_decode_kernel<BR, TR, BS, TS, LOOP><<<grid, kLayerThreads, lds_bytes, st>>>(a);
    return FATE_OK;
}
// workgroups of one kernel variant that fit on a compute unit with lds_bytes of dynamic LDS (0: the query failed)
template <int BR, int TR, int BS, int TS, bool LOOP>
static int layer_kernel_blocks_per_cu(int lds_bytes, int lds_max) {
    const void* f = reinterpret_cast<const void*>(moe_layer_decode_kernel<BR, TR, BS, TS, LOOP>);
    if (hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lds_max) != hipSuccess) return 0;
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, f, kLayerThreads, (size_t)lds_bytes) != hipSuccess) return 0;
    return nb;
}
template <int BR, int TR, bool LOOP>
static int layer_routed_blocks_per_cu(int bits_s, int tpg_s, int lds_bytes, int lds_max) {
    int nb = 0;
#define FATE_SHARED_BODY(BS, TS) nb = layer_kernel_blocks_per_cu<BR, TR, BS, TS, LOOP>(lds_bytes, lds_max);
    FATE_FORMAT_SWITCH(bits_s, tpg_s, FATE_SHARED_BODY)
#undef FATE_SHARED_BODY
    return nb;
}

template <int BR, int TR, bool LOOP>
static fate_status launch_layer_routed(hipStream_t st, int bits_s, int tpg_s, int grid, int lds_bytes, int lds_max,
                                       const LayerArgs& a) {
    fate_status rc = FATE_OK;
#define FATE_SHARED_BODY(BS, TS) rc = launch_layer_kernel_v<BR, TR, BS, TS, LOOP>(st, grid, lds_bytes, lds_max, a);
    FATE_FORMAT_SWITCH(bits_s, tpg_s, FATE_SHARED_BODY)
#undef FATE_SHARED_BODY
    return rc;
}

}  // namespace fate
