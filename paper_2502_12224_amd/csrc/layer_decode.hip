// fate_moe_layer_decode: one launch for a whole decode-side MoE layer (1..8
// tokens): gate logits, softmax / top-k, cross-layer prediction, permutation
// and the quantised expert FFN.
//
// Block ids, in order:
//  routing workgroups: each wave evaluates one gate row (this layer's gate,
//    then the next layer's) for every token and publishes the logit tagged
//    with the call's epoch.  The first of them also clear y.  The last one
//    waits for all logits and writes the routing outputs of the API.
//  work blocks: 64 intermediate neurons of one shared expert or of one routed
//    slot.  A routed block polls the tagged logits (the only cross-workgroup
//    dependency on its path), redoes softmax / top-k / permutation for itself
//    in LDS - same code on the same bits as the routing workgroup - and so
//    learns its expert without waiting for another workgroup's bookkeeping.
//    Then: all requests for its W1/W3 row blocks and W2 column block go out,
//    eight waves split the reduction dimension of the up projection, the 64
//    values of h stay in LDS, and each wave multiplies them into its share of
//    the 32-row blocks of W2 and adds weight * partial into y with fp32
//    atomics (blocks walk the row blocks from different starting points so
//    that they do not hit the same addresses at the same time).
// A workgroup only ever waits for workgroups with lower ids, which the
// dispatcher of its compute die has started before it; every wait is bounded
// and turns into a status bit when it runs out.
#include <hip/hip_fp16.h>
#include "common.h"
#include "qformat.h"
#include "decode_device.h"
#include "route_device.h"
#include "layer_decode.h"

namespace fate {

constexpr int kSpinMax = 1 << 18;
constexpr int kUpRing = 4;        // tiles in flight per (row block, matrix) per wave: 16 KiB
constexpr int kDownRing = 8;      // W2 tiles in flight per wave
constexpr int kHsLd = kLayerNeurons + kLdsPad;   // halves per row of h in LDS

#ifdef FATE_PROBE
// Timing probes (builds with -DFATE_PROBE only): per workgroup eight 100 MHz
// timestamps, read back with fate_debug_probe().
__device__ unsigned long long g_probe[4096 * 8];
#define FATE_TS(i) do { if (threadIdx.x == 0 && blockIdx.x < 4096) g_probe[blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
#else
#define FATE_TS(i) do { } while (0)
#endif

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

// LDS carve of a work block (bytes from the start of dynamic shared memory)
struct WorkLds {
    int xs, hs, red, tab, zl, ids, w, counts, offsets, perm, inv, order, tokid, wtok, bytes;
};
__host__ __device__ inline WorkLds work_lds(int N, int H, int E, int k) {
    auto up = [](int v) { return (v + 15) & ~15; };
    const int ntp = N < kTokPass ? N : kTokPass;
    const int P = N * k;
    WorkLds L;
    int off = 0;
    L.xs = off; off += up((N + 1) * (H + kLdsPad) * 2);
    L.hs = off; off += up((kTokPass + 1) * kHsLd * 2);
    L.red = off; off += up(kLayerWaves * 4 * ntp * 32 * 4);
    L.tab = off; off += up(E * (int)sizeof(fate_qexpert));
    L.zl = off; off += up(2 * N * E * 4);
    L.ids = off; off += up(P * 4);
    L.w = off; off += up(P * 4);
    L.counts = off; off += up(E * 4);
    L.offsets = off; off += up((E + 1) * 4);
    L.perm = off; off += up(P * 4);
    L.inv = off; off += up(P * 4);
    L.order = off; off += up(E * 4);
    L.tokid = off; off += up(kTokPass * 4);
    L.wtok = off; off += up(kTokPass * 4);
    L.bytes = off;
    return L;
}

__device__ __forceinline__ void route_role(const LayerArgs& a, int b, uint32_t tag, char* dyn, FusedRouteSmem& rsm) {
    const int tid = threadIdx.x;
    const FusedRouteArgs& r = a.r;
    if (b < a.nb_zero) {
        const int total = r.N * r.H;
        const int per = (total + a.nb_zero - 1) / a.nb_zero;
        const int b1 = min(total, (b + 1) * per);
        for (int i = b * per + tid; i < b1; i += kLayerThreads) st_dev(a.y + i, 0.f);
        // the cleared slice is in place before any logit of this workgroup can be seen
        __syncthreads();
    }
    fused_gate_rows(r, b, TaggedStore{a.zq, r.N, r.E, tag});
    FATE_TS(1);
    if (b != a.nb_route - 1) return;
    // the routing outputs of the API (consumers inside this launch do not read them)
    float* zl = reinterpret_cast<float*>(dyn);
    const int n = (r.Wg2 ? 2 : 1) * r.N * r.E;
    if (!wait_logits(a.zq, n, tag, zl)) {
        if (tid == 0) atomicOr(a.status, 2);
        return;
    }
    FATE_TS(2);
    fused_select(r, rsm, nullptr, LdsLoad{zl, r.N, r.E});
    FATE_TS(3);
}

__device__ __forceinline__ void work_role(const LayerArgs& a, int wb, uint32_t tag, char* dyn) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
    const bool defer_x = is_shared && x_one;
    if (!defer_x) store_x(false);

    fate_qexpert ex;
    int kb, T, bits, group;
    if (is_shared) {
        const int s = wb / a.nkb_s;
        kb = wb - s * a.nkb_s;
        ex = a.shared[s];
        T = N;
        bits = a.bits_s; group = a.group_s;
        if (a.shared_gate != nullptr) {
            for (int t = wave; t < N; t += kLayerWaves) {
                const float g = wave_sigmoid_dot_bf16(reinterpret_cast<const uint4*>(a.r.x) + (size_t)t * nvec,
                                                      reinterpret_cast<const uint4*>(a.shared_gate), nvec);
                if (lane == 0) wtok[t] = g;
            }
        } else if (tid < N) {
            wtok[tid] = 1.0f;
        }
        if (tid < N) tokid[tid] = tid;
    } else {
        uint4* tab = reinterpret_cast<uint4*>(dyn + L.tab);
        float* zl = reinterpret_cast<float*>(dyn + L.zl);
        int32_t* ids = reinterpret_cast<int32_t*>(dyn + L.ids);
        float* wv = reinterpret_cast<float*>(dyn + L.w);
        int32_t* counts = reinterpret_cast<int32_t*>(dyn + L.counts);
        int32_t* offsets = reinterpret_cast<int32_t*>(dyn + L.offsets);
        int32_t* perm = reinterpret_cast<int32_t*>(dyn + L.perm);
        int32_t* inv = reinterpret_cast<int32_t*>(dyn + L.inv);
        int32_t* order = reinterpret_cast<int32_t*>(dyn + L.order);
        // the expert table travels while the logits are awaited
        {
            const uint4* src = reinterpret_cast<const uint4*>(a.experts);
            for (int i = tid; i < E * (int)(sizeof(fate_qexpert) / 16); i += kLayerThreads) tab[i] = src[i];
        }
        if (!wait_logits(a.zq, N * E, tag, zl)) {
            if (tid == 0) atomicOr(a.status, 2);
            return;
        }
        FATE_TS(1);
        if (wave < N)
            wave_softmax_topm(zl + wave * E, E, k, a.r.renorm, ids + wave * k, wv + wave * k, nullptr, nullptr);
        __syncthreads();
        if (wave == 0) wave_permute_small(ids, N * k, E, counts, offsets, perm, inv, order);
        __syncthreads();
        const int rwb = wb - nsh;
        const int slot = rwb / a.nkb_r;
        kb = rwb - slot * a.nkb_r;
        const int e = order[slot];
        T = counts[e];
        if (T == 0) return;
        const int sbeg = offsets[e];
        ex = reinterpret_cast<const fate_qexpert*>(tab)[e];
        bits = a.bits_r; group = a.group_r;
        if (tid < T) {
            const int p = perm[sbeg + tid];
            tokid[tid] = p / k;
            wtok[tid] = wv[p];
        }
    }
    const int I = ex.I;
    if (kb * kLayerNeurons >= I) return;
    if (ex.w1 == nullptr || ex.w3 == nullptr || ex.w2 == nullptr) {
        if (tid == 0) atomicOr(a.status, 1);
        return;
    }
    const int KT = bits == 4 ? 64 : 32;
    const int tpg = group / KT;
    const int G = H / group;                 // groups along the reduction dimension of W1 / W3
    const int tiles_k = H / KT;
    const int g_beg = G * wave / kLayerWaves, g_end = G * (wave + 1) / kLayerWaves;
    gu4_t wt[4];
    gu16_t sc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int rb = 2 * kb + (i >> 1);
        wt[i] = as_global<uint4>((i & 1) ? ex.w3 : ex.w1) + (size_t)rb * tiles_k * 64 + lane;
        sc[i] = as_global<uint16_t>((i & 1) ? ex.s3 : ex.s1) + (size_t)(rb * 32 + n) * G;
    }
    // W2: the column block [kb*64, kb*64+64) of every 32-row block; this wave takes row blocks
    // wave, wave+8, ... starting from a block-dependent one
    const int tpn = kLayerNeurons / KT;      // tiles per row block: 1 (int4) or 2 (int8)
    const int tiles_k2 = I / KT;
    const int G2 = I / group, g2 = kb * kLayerNeurons / group;
    const int nrb = H >> 5;
    const int nq = (nrb - wave + kLayerWaves - 1) / kLayerWaves;     // row blocks of this wave
    const int qrot = nq > 0 ? wb % nq : 0;
    gu4_t w2 = as_global<uint4>(ex.w2) + (size_t)kb * tpn * 64 + lane;
    gu16_t s2 = as_global<uint16_t>(ex.s2) + (size_t)n * G2 + g2;
    auto rb_of = [&](int q) { int qq = q + qrot; if (qq >= nq) qq -= nq; return wave + kLayerWaves * qq; };

#define FATE_LAYER_BODY(BITS, TPG)                                                                        \
    {                                                                                                     \
        constexpr int S = QFmt<BITS>::MSTEPS, TPN = kLayerNeurons / QFmt<BITS>::KT;                       \
        if (defer_x) load_x();                                                                            \
        TileRing<4, kUpRing, TPG> ring;                                                                   \
        ring_start<4, kUpRing, TPG>(ring, wt, sc, g_beg, g_end);                                          \
        /* W2 tiles behind them */                                                                        \
        uint4 draw[kDownRing];                                                                            \
        uint32_t dsc[kDownRing / TPN];                                                                    \
        const int nu = nq * TPN;                                                                          \
        _Pragma("unroll")                                                                                 \
        for (int u = 0; u < kDownRing; ++u) {                                                             \
            if (u < nu) {                                                                                 \
                const int rb = rb_of(u / TPN);                                                            \
                draw[u] = w2[((size_t)rb * tiles_k2 + (u % TPN)) * 64];                                   \
                if (u % TPN == 0) dsc[u / TPN] = s2[(size_t)rb * 32 * G2];                                \
            }                                                                                             \
        }                                                                                                 \
        if (defer_x) store_x(true);                                                                       \
        /* y must have been cleared before this block adds to it: every logit of this layer's gate  */   \
        /* carries that guarantee (a routed block has waited for them already)                      */   \
        if (is_shared && !wait_logits(a.zq, N * E, tag, reinterpret_cast<float*>(dyn + L.zl))) {          \
            if (tid == 0) atomicOr(a.status, 2);                                                          \
            return;                                                                                       \
        }                                                                                                 \
        __syncthreads();          /* x, token ids and weights are in LDS */                               \
        FATE_TS(2);                                                                                       \
        float out[4][4];                                                                                  \
        _Pragma("unroll")                                                                                 \
        for (int i = 0; i < 4; ++i)                                                                       \
            _Pragma("unroll")                                                                             \
            for (int j = 0; j < 4; ++j) out[i][j] = 0.f;                                                  \
        const int arow = n < T ? tokid[n] : N;                                                            \
        ring_run<BITS, TPG, 4, kUpRing>(ring, wt, sc, g_beg, g_end,                                       \
                                        xs + arow * ldx + half * (QFmt<BITS>::KT / 2), 0, out);           \
        FATE_TS(3);                                                                                       \
        _Pragma("unroll")                                                                                 \
        for (int i = 0; i < 4; ++i)                                                                       \
            _Pragma("unroll")                                                                             \
            for (int j = 0; j < 4; ++j)                                                                   \
                if (4 * half + j < ntp) red[((wave * 4 + i) * ntp + 4 * half + j) * 32 + n] = out[i][j];  \
        __syncthreads();                                                                                  \
        for (int idx = tid; idx < T * kLayerNeurons; idx += kLayerThreads) {                              \
            const int t = idx >> 6, nn = idx & 63, sel = nn >> 5, n32 = nn & 31;                          \
            float a1 = 0.f, a3 = 0.f;                                                                     \
            _Pragma("unroll")                                                                             \
            for (int w = 0; w < kLayerWaves; ++w) {                                                       \
                a1 += red[((w * 4 + 2 * sel) * ntp + t) * 32 + n32];                                      \
                a3 += red[((w * 4 + 2 * sel + 1) * ntp + t) * 32 + n32];                                  \
            }                                                                                             \
            hs[t * kHsLd + nn] = (_Float16)(a1 / (1.0f + expf(-a1)) * a3);                                \
        }                                                                                                 \
        __syncthreads();                                                                                  \
        FATE_TS(4);                                                                                       \
        /* down projection of the 64 values of h */                                                       \
        const _Float16* ha = hs + (n < T ? n : kTokPass) * kHsLd + half * (QFmt<BITS>::KT / 2);           \
        float wj[4];                                                                                      \
        int tj[4];                                                                                        \
        _Pragma("unroll")                                                                                 \
        for (int j = 0; j < 4; ++j) {                                                                     \
            const int t = 4 * half + j;                                                                   \
            wj[j] = t < T ? wtok[t] : 0.f;                                                                \
            tj[j] = t < T ? tokid[t] : 0;                                                                 \
        }                                                                                                 \
        const f32x16_t zero = f32x16_zero();                                                              \
        for (int base = 0; base < nu; base += kDownRing) {                                                \
            _Pragma("unroll")                                                                             \
            for (int uq = 0; uq < kDownRing / TPN; ++uq) {                                                \
                if (base + uq * TPN < nu) {                                                               \
                    const int q = (base + uq * TPN) / TPN;                                                \
                    const int rb = rb_of(q);                                                              \
                    const float s = half_bits_to_float(dsc[uq]);                                          \
                    const int qn = q + kDownRing / TPN;                                                   \
                    if (qn < nq) dsc[uq] = s2[(size_t)rb_of(qn) * 32 * G2];                               \
                    f32x16_t acc;                                                                         \
                    _Pragma("unroll")                                                                     \
                    for (int sub = 0; sub < TPN; ++sub) {                                                 \
                        const int u = uq * TPN + sub;                                                     \
                        f16x8_t bq[S];                                                                    \
                        codes_to_f16<BITS>(draw[u], bq);                                                  \
                        if (qn < nq) draw[u] = w2[((size_t)rb_of(qn) * tiles_k2 + sub) * 64];             \
                        _Pragma("unroll")                                                                 \
                        for (int st = 0; st < S; ++st) {                                                  \
                            const f16x8_t av = *reinterpret_cast<const f16x8_t*>(                         \
                                ha + sub * QFmt<BITS>::KT + 8 * st);                                      \
                            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(                                 \
                                av, bq[st], (sub == 0 && st == 0) ? zero : acc, 0, 0, 0);                 \
                        }                                                                                 \
                    }                                                                                     \
                    _Pragma("unroll")                                                                     \
                    for (int j = 0; j < 4; ++j)                                                           \
                        if (4 * half + j < T)                                                             \
                            atomicAdd(a.y + (size_t)tj[j] * H + rb * 32 + n, wj[j] * (s * acc[j]));       \
                }                                                                                         \
            }                                                                                             \
        }                                                                                                 \
    }
    FATE_FORMAT_SWITCH(bits, tpg, FATE_LAYER_BODY)
#undef FATE_LAYER_BODY
}

__global__ __launch_bounds__(kLayerThreads) void moe_layer_decode_kernel(LayerArgs a) {
    extern __shared__ uint4 smem[];
    __shared__ FusedRouteSmem rsm;
    char* dyn = reinterpret_cast<char*>(smem);
    uint32_t tag = (uint32_t)ld_dev(a.sync) + 1u;
    if (tag == 0u) tag = 1u;         // a zero-filled workspace must never look current
    FATE_TS(0);
    const int b = blockIdx.x;
    if (b < a.nb_route) route_role(a, b, tag, dyn, rsm);
    else work_role(a, b - a.nb_route, tag, dyn);
    // the workgroup that leaves last opens the next epoch
    __syncthreads();
    FATE_TS(7);
    if (threadIdx.x == 0 && atomicAdd(a.sync + 1, 1) == (int)gridDim.x - 1) {
        st_dev(a.sync + 1, 0);
        st_dev(a.sync, (int32_t)tag);
    }
}

__global__ void layer_f32_to_bf16_kernel(const float* __restrict__ src, uint16_t* __restrict__ dst, long long n) {
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = (uint16_t)f32_to_bf16_bits(src[i]);
}

#ifdef FATE_PROBE
extern "C" int fate_debug_probe(unsigned long long* host_out, int nblocks) {
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(g_probe), (size_t)nblocks * 8 * sizeof(unsigned long long));
}
#endif

fate_status launch_layer_decode(hipStream_t st, const fate_ffn_desc& d, LayerArgs a, void* y_out) {
    if (d.N < 1 || d.N > kLayerMaxN || d.N * d.k > kLayerMaxP)
        FATE_FAIL(FATE_ESHAPE, "fused layer: need 1 <= N <= %d and N*k <= %d (N = %d, k = %d)", kLayerMaxN,
                  kLayerMaxP, d.N, d.k);
    if (!decode_group_ok(d.bits, d.group) || (d.n_shared && !decode_group_ok(d.shared_bits, d.shared_group)))
        FATE_FAIL(FATE_ESHAPE, "fused layer: group must be 64, 128 or 256 (int4) / 64 or 128 (int8)");
    const WorkLds L = work_lds(d.N, d.H, d.E, d.k);
    constexpr int kLdsMax = 128 * 1024;
    if (L.bytes > kLdsMax) FATE_FAIL(FATE_ESHAPE, "fused layer: N = %d, H = %d need %d bytes of LDS", d.N, d.H, L.bytes);
    static bool attr_done = false;
    if (!attr_done) {
        FATE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(moe_layer_decode_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kLdsMax));
        attr_done = true;
    }
    const int rows = (a.r.Wg2 ? 2 : 1) * d.E;
    a.nb_route = (rows + kLayerWaves - 1) / kLayerWaves;
    a.nb_zero = (d.E + kLayerWaves - 1) / kLayerWaves;        // the workgroups that hold this layer's gate rows
    a.nkb_r = d.I_max / kLayerNeurons;
    a.nkb_s = d.n_shared ? d.I_shared_max / kLayerNeurons : 0;
    a.nact = min(d.E, d.N * d.k);
    const int grid = a.nb_route + d.n_shared * a.nkb_s + a.nact * a.nkb_r;
    moe_layer_decode_kernel<<<grid, kLayerThreads, L.bytes, st>>>(a);
    FATE_HIP(hipGetLastError());
    if (!d.y_is_fp32) {
        const long long n = (long long)d.N * d.H;
        layer_f32_to_bf16_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(a.y, static_cast<uint16_t*>(y_out), n);
        FATE_HIP(hipGetLastError());
    }
    return FATE_OK;
}

}  // namespace fate
