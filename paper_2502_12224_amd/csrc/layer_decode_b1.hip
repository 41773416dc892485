// fate_moe_layer_decode for one token: one launch, no partial output rows.
//
// Block ids, in order:
//   routing blocks      gate rows of this layer and of the next one, logits published as
//                       epoch-tagged words; the last one writes the API's routing outputs
//   shared up blocks    32 intermediate neurons of a shared expert: W1 / W3 row block, SwiGLU,
//                       h published as tagged pairs of fp16
//   routed up blocks    as the shared ones, after polling the logits and finding the slot's expert
//                       (slot j = the expert with the j-th largest logit)
//   down blocks         32 output rows: each wave fetches a K range of W2 of a shared expert at once
//                       and a K range of W2 of a routed slot as soon as the selection is known,
//                       polls the shared h of its range and multiplies, then the routed h; the
//                       block publishes a tagged partial output, and the last block of an output
//                       row block polls the other blocks' partial outputs, adds them in a fixed
//                       order and writes y
// Every wait is on data of blocks with lower ids, bounded, and turns into status bit 1.
// Requests that do not depend on the routing (shared W1 / W3 / W2) all go out at the start;
// W2 of the routed experts goes out as soon as a down block knows the selection, long before
// the routed h exists; when it exists, half of every down wave's products are already done.
#include "layer_decode_impl.h"
#include "layer_decode_b1.h"

namespace fate {


// ---- LDS of a down block -----------------------------------------------------------------
constexpr int kB1HRegion = kB1MaxTiles * 64;          // halves of h per wave (tiles of at most 64 columns)
struct B1DownLds {
    int hl, zrow, red, red2, tab, zl, ids, w, src_e, src_w, gate, bytes;
};
__host__ __device__ inline B1DownLds b1_down_lds(int E, int k) {
    auto up = [](int v) { return (v + 15) & ~15; };
    B1DownLds L;
    int off = 0;
    L.hl = off; off += up(kLayerWaves * kB1HRegion * 2);
    L.zrow = off; off += up(kB1HRegion * 2);
    L.red = off; off += up(kLayerWaves * 32 * 4);
    L.red2 = off; off += up(kLayerWaves * 32 * 4);
    L.tab = off; off += up(E * (int)sizeof(fate_qexpert));
    L.zl = off; off += up(2 * E * 4);
    L.ids = off; off += up(k * 4);
    L.w = off; off += up(k * 4);
    L.src_e = off; off += up(k * 4);
    L.src_w = off; off += up(k * 4);
    L.gate = off; off += 16;
    L.bytes = off;
    return L;
}

// ---- up block: 32 neurons of one expert, one token -----------------------------------------
// The straight-line up projection of the general kernel (register ring, codes + constant on the
// matrix cores, constant removed per group) in two steps, so that the requests can be in flight
// while the block does something else: b1_up_issue asks for the first ring of W1 / W3 tiles and
// their scales, b1_up_compute multiplies and returns, in lanes 0..31 of wave 0, the fp16 bits of
// h of neuron kb*32 + lane.
template <int TPG>
struct B1UpRegs {
    uint4 raw[2][kUpRing];
    uint32_t scr[2][kUpRing / TPG];
};

template <int BITS, int TPG>
struct B1UpAddr {
    gu4_t wt[2];
    gu16_t sc[2];
    int g_beg, tw;
    __device__ __forceinline__ B1UpAddr(const WorkCtx& c) {
        constexpr int KT = QFmt<BITS>::KT;
        const int lane = c.tid & 63, wave = __builtin_amdgcn_readfirstlane(c.tid >> 6);
        const int n = lane & 31;
        const int tiles_k = c.H / KT;
        tw = tiles_k / kLayerWaves;
        g_beg = wave * (tw / TPG);
        wt[0] = as_global<uint4>(c.ex.w1) + ((size_t)c.kb * tiles_k + wave * tw) * 64 + lane;
        wt[1] = as_global<uint4>(c.ex.w3) + ((size_t)c.kb * tiles_k + wave * tw) * 64 + lane;
        sc[0] = as_global<uint16_t>(c.ex.s1) + (size_t)g_beg * c.I + c.kb * 32 + n;
        sc[1] = as_global<uint16_t>(c.ex.s3) + (size_t)g_beg * c.I + c.kb * 32 + n;
    }
};

template <int BITS, int TPG, class LoadX>
__device__ __forceinline__ void b1_up_issue(const WorkCtx& c, B1UpRegs<TPG>& R, LoadX&& load_x) {
    constexpr int D = kUpRing, GR = D / TPG;
    const B1UpAddr<BITS, TPG> ad(c);
    if (c.defer_x) load_x();
#pragma unroll
    for (int j = 0; j < D; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i) R.raw[i][j] = ad.wt[i][(size_t)j * 64];
#pragma unroll
    for (int jg = 0; jg < GR; ++jg)
#pragma unroll
        for (int i = 0; i < 2; ++i) R.scr[i][jg] = ad.sc[i][(size_t)jg * c.I];
}

template <int BITS, int TPG, class StoreX>
__device__ __forceinline__ uint32_t b1_up_compute(const WorkCtx& c, B1UpRegs<TPG>& R, StoreX&& store_x) {
    constexpr int KT = QFmt<BITS>::KT, D = kUpRing;
    const int tid = c.tid, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, half = lane >> 5;
    const B1UpAddr<BITS, TPG> ad(c);
    const int tw = ad.tw, g_beg = ad.g_beg, I = c.I;
    const int rounds = tw / D;
    if (c.defer_x) store_x(true);
    lds_barrier();            // x and the zero row are in LDS
    {   // sums of x times the codes' constant for this wave's groups: 8 lanes per token row
        constexpr int per = KT * TPG / 8;
        const int t = lane >> 3, sub = lane & 7;
        const _Float16* xp = c.xs + (t < 1 ? t : 1) * c.ldx + (size_t)g_beg * (KT * TPG) + sub * per;
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
    const int arow = n < 1 ? 0 : 1;                  // row 0 = the token, row 1 = zeros
    int ctok[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) ctok[j] = 4 * half + j < 1 ? 0 : kTokPass;
    const _Float16* xa = c.xs + arow * c.ldx + half * (KT / 2) + (size_t)wave * tw * KT;
    const float* cxg = c.cx + g_beg * kCxLd;
    for (int r = 0; r + 1 < rounds; ++r)
        up_round<BITS, TPG, true>(R.raw, R.scr, ad.wt, ad.sc, I, r, xa, cxg, ctok, bc, out, [] {});
    up_round<BITS, TPG, false>(R.raw, R.scr, ad.wt, ad.sc, I, rounds - 1, xa, cxg, ctok, bc, out, [] {});
    if (half == 0) {
        c.red[(wave * 2 + 0) * 32 + n] = out[0][0];
        c.red[(wave * 2 + 1) * 32 + n] = out[1][0];
    }
    lds_barrier();
    uint32_t mine = 0;
    if (tid < 32) {
        float a1 = 0.f, a3 = 0.f;
#pragma unroll
        for (int w = 0; w < kLayerWaves; ++w) {
            a1 += c.red[(w * 2) * 32 + n];
            a3 += c.red[(w * 2 + 1) * 32 + n];
        }
        const _Float16 hv = (_Float16)(a1 / (1.0f + expf(-a1)) * a3);
        mine = (uint32_t)__builtin_bit_cast(unsigned short, hv);
    }
    return mine;
}

// 32 values of h (fp16 bits in lanes 0..31 of wave 0) go out as 16 tagged words
__device__ __forceinline__ void b1_publish_h(unsigned long long* hq_dst, uint32_t tag, uint32_t mine) {
    if (threadIdx.x < 32) {
        const uint32_t next = (uint32_t)__shfl_down((int)mine, 1, 64);
        if ((threadIdx.x & 1) == 0)
            __hip_atomic_store(hq_dst + (threadIdx.x >> 1),
                               ((unsigned long long)tag << 32) | (unsigned long long)(mine | (next << 16)),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Routed blocks: poll the logits, redo softmax / top-k (wave 0), leave ids and weights in LDS.
// The expert table travels to LDS while the logits are awaited.
// Which expert each routed slot works on.  Without a hint slot j takes the expert of rank j.
// With a hint (k expert ids predicted for this layer, from the previous layer's call) the
// blocks of slot j have started on expert hint[j] before the gate was known: slot j keeps it
// if it is among the selected ones (first occurrence only), and the selected experts that
// no slot holds go, in rank order, to the slots whose hint missed.  One wave; k <= 64.
__device__ __forceinline__ void b1_assign_slots(const int32_t* hint, const int32_t* ids, int k, int E, int32_t* src_e,
                                                int32_t* src_r) {
    const int lane = threadIdx.x & 63;
    const int mine = lane < k ? ids[lane] : -1;          // lane r: the expert of rank r
    int hj = -1;
    if (hint != nullptr && lane < k) {
        hj = hint[lane];
        if (hj < 0 || hj >= E) hj = -1;
    }
    int rank_of_hint = -1;                                // slot `lane`: rank of its hinted expert, if selected
    bool dup = false;
    for (int r = 0; r < k; ++r) {
        const int er = lane_bcast(mine, r), hr = lane_bcast(hj, r);
        if (hj >= 0 && er == hj) rank_of_hint = r;
        if (r < lane && hr == hj) dup = true;
    }
    const bool hit = lane < k && hj >= 0 && rank_of_hint >= 0 && !dup;
    const unsigned long long hitmask = __ballot(hit);
    bool taken = false;                                   // lane r: does a hit slot hold the expert of rank r?
    for (int j = 0; j < k; ++j) {
        const int rj = lane_bcast(rank_of_hint, j);
        if (((hitmask >> j) & 1ull) && rj == lane) taken = true;
    }
    const unsigned long long freemask = __ballot(lane < k && !taken);    // ranks still to be placed
    int r_mine = rank_of_hint;
    if (lane < k && !hit) {
        int nth = __popcll(~hitmask & ((1ull << lane) - 1ull));           // this slot is the nth missing one
        unsigned long long fm = freemask;
        for (int i = 0; i < nth; ++i) fm &= fm - 1;                       // drop the nth lowest set bits
        r_mine = __ffsll((long long)fm) - 1;
    }
    const int e_mine = __shfl(mine, r_mine < 0 ? 0 : r_mine, 64);
    if (lane < k) {
        src_e[lane] = e_mine;
        src_r[lane] = r_mine < 0 ? 0 : r_mine;        // its rank: where the selection's weights will hold its weight
    }
}

// Routed blocks: wait for the logits (the expert table travels to LDS meanwhile) and find the
// expert of the block's slot - ids only, no softmax: the selection's weights are needed much later
// and only by the down blocks.  Without a hint every wave finds the expert of rank `slot` by itself;
// with a hint wave 0 takes all k ranks, matches them against the hinted experts and the other
// waves read the result after one LDS barrier.  Returns false when the wait ran out.
__device__ __forceinline__ bool b1_slot_expert(const B1Args& A, uint32_t tag, int slot, uint4* tab, float* zl, int32_t* ids,
                                               int32_t* src_e, int32_t* src_r, int* e_true, int* rank) {
    const LayerArgs& a = A.a;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int E = a.r.E;
    const uint4* src = reinterpret_cast<const uint4*>(a.experts);
    for (int i = tid; i < E * (int)(sizeof(fate_qexpert) / 16); i += kLayerThreads) tab[i] = src[i];
    if (!wait_logits(a.zq, E, tag, zl)) {
        if (tid == 0) atomicOr(a.status, 2);
        return false;
    }
    if (a.hint == nullptr) {
        *e_true = __builtin_amdgcn_readfirstlane(wave_rank_expert(zl, E, slot));
        *rank = slot;
        return true;
    }
    if (wave == 0) {
        wave_topk_ids(zl, E, a.r.k, ids);
        __builtin_amdgcn_wave_barrier();
        b1_assign_slots(a.hint, ids, a.r.k, E, src_e, src_r);
    }
    lds_barrier();
    *e_true = src_e[slot];
    *rank = src_r[slot];
    return true;
}

__device__ __forceinline__ bool b1_entry_usable(const fate_qexpert& ex, int bits, int group) {
    return ex.w1 != nullptr && ex.w3 != nullptr && ex.w2 != nullptr && ex.bits == bits && ex.group == group &&
           ex.z1 == nullptr;
}

template <int BR, int TR, int BS, int TS, bool HINTED>
__device__ __forceinline__ void b1_up_role(const B1Args& A, int ub, bool is_shared, uint32_t tag, char* dyn) {
    const LayerArgs& a = A.a;
    const int tid = threadIdx.x;
    const int H = a.r.H, E = a.r.E, k = a.r.k;
    const WorkLds L = work_lds(1, H, E, k);
    _Float16* xs = reinterpret_cast<_Float16*>(dyn + L.xs);
    const int ldx = H + kLdsPad, nvec = H >> 3;
    const bool x_one = nvec <= kLayerThreads;
    uint4 xv = make_uint4(0, 0, 0, 0);
    auto load_x = [&]() {
        if (tid < nvec) xv = reinterpret_cast<const uint4*>(a.r.x)[tid];
    };
    auto store_x = [&](bool from_reg) {
        if (from_reg) {
            if (tid < nvec) *reinterpret_cast<uint4*>(xs + tid * 8) = bf16x8_to_f16x8(xv);
        } else {
            const uint4* xg = reinterpret_cast<const uint4*>(a.r.x);
            for (int idx = tid; idx < nvec; idx += kLayerThreads)
                *reinterpret_cast<uint4*>(xs + idx * 8) = bf16x8_to_f16x8(xg[idx]);
        }
        for (int c = tid; c < (ldx >> 3); c += kLayerThreads)
            *reinterpret_cast<uint4*>(xs + ldx + c * 8) = make_uint4(0, 0, 0, 0);
    };
    const bool defer_x = is_shared && x_one;
    if (!defer_x) store_x(false);

    WorkCtx cx;
    cx.tid = tid;
    cx.N = 1; cx.H = H; cx.T = 1; cx.wb = ub; cx.ntp = 1; cx.ldx = ldx;
    cx.is_shared = is_shared; cx.defer_x = defer_x; cx.xs = xs;
    cx.hs = reinterpret_cast<_Float16*>(dyn + L.hs);
    cx.red = reinterpret_cast<float*>(dyn + L.red);
    cx.wtok = nullptr; cx.cx = reinterpret_cast<float*>(dyn + L.cx); cx.ch = nullptr;
    cx.tokid = nullptr; cx.pairq = nullptr; cx.part = nullptr; cx.part_stride = 0;
    if (is_shared) {
        const int s = ub / a.nkb_s;
        const int kb = ub - s * a.nkb_s;
        unsigned long long* hq_dst = A.a.hq + ((size_t)s * a.nkb_s + kb) * 16;
        const fate_qexpert ex = a.shared[s];
        const bool absent = !b1_entry_usable(ex, a.bits_s, a.group_s);
        uint32_t hbits = 0;
        if (absent && tid == 0) atomicOr(a.status, 1);
        if (!absent && kb * kLayerNeurons < ex.I) {
            cx.I = ex.I; cx.kb = kb; cx.ex = ex;
            B1UpRegs<TS> R;
            b1_up_issue<BS, TS>(cx, R, load_x);
            hbits = b1_up_compute<BS, TS>(cx, R, store_x);
        }
        b1_publish_h(hq_dst, tag, hbits);
        return;
    }
    // Routed slot.  With a hint (the paper's cross-layer prediction used as a prefetch: section 4.3)
    // the requests for the hinted expert go out before the gate is known; once the logits are there
    // the block checks the hint against the gate's selection and asks again only if it was wrong.
    const int slot = ub / a.nkb_r;
    const int kb = ub - slot * a.nkb_r;
    unsigned long long* hq_dst = A.a.hq + ((size_t)a.n_shared * a.nkb_s + (size_t)slot * a.nkb_r + kb) * 16;
    uint4* tab = reinterpret_cast<uint4*>(dyn + L.tab);
    float* zl = reinterpret_cast<float*>(dyn + L.zl);
    int32_t* ids = reinterpret_cast<int32_t*>(dyn + L.ids);
    int32_t* src_e = reinterpret_cast<int32_t*>(dyn + L.pairq);     // (regions the one-token kernel has no other use for)
    int32_t* src_r = reinterpret_cast<int32_t*>(dyn + L.wtok);
    B1UpRegs<TR> R;
    int e_cur = -1;
    bool in_flight = false;                 // requests for expert e_cur are under way
    if constexpr (HINTED) {
        e_cur = a.hint[slot];
        if (e_cur < 0 || e_cur >= E) e_cur = -1;
        if (e_cur >= 0) {
            const fate_qexpert ex = a.experts[e_cur];
            if (b1_entry_usable(ex, a.bits_r, a.group_r) && kb * kLayerNeurons < ex.I) {
                cx.I = ex.I; cx.kb = kb; cx.ex = ex;
                b1_up_issue<BR, TR>(cx, R, load_x);
                in_flight = true;
            }
        }
    }
    int e_true = -1, rank = 0;
    if (!b1_slot_expert(A, tag, slot, tab, zl, ids, src_e, src_r, &e_true, &rank)) {
        b1_publish_h(hq_dst, tag, 0);
        return;
    }
    bool ready = in_flight && e_true == e_cur;
    if (!ready && e_true >= 0) {
        const fate_qexpert ex = reinterpret_cast<const fate_qexpert*>(tab)[e_true];
        const bool usable = b1_entry_usable(ex, a.bits_r, a.group_r);
        if (!usable && tid == 0) atomicOr(a.status, 1);
        if (usable && kb * kLayerNeurons < ex.I) {
            cx.I = ex.I; cx.kb = kb; cx.ex = ex;
            b1_up_issue<BR, TR>(cx, R, load_x);
            ready = true;
        }
    }
    uint32_t hbits = 0;
    if (ready) hbits = b1_up_compute<BR, TR>(cx, R, store_x);
    b1_publish_h(hq_dst, tag, hbits);
}

// ---- down block: 32 output rows, four wave items --------------------------------------------
// Requests of one wave item: its W2 tiles of output row block rb and their scales.  Returns the
// number of groups the expert really has in the item's range (0: nothing requested).
template <int BITS, int TPG>
__device__ __forceinline__ int b1_down_request(const fate_qexpert& ex, int H, int rb, int g0, int ng,
                                               uint4 (&raw)[kB1MaxTiles], uint32_t (&sc)[kB1MaxTiles / TPG]) {
    constexpr int KT = QFmt<BITS>::KT, MAXG = kB1MaxTiles / TPG;
    const int lane = threadIdx.x & 63;
    const int n = lane & 31;
    const int group = KT * TPG;
    const int tiles_k2 = ex.I / KT;
    const int gmax = ex.I / group;
    ng = g0 + ng <= gmax ? ng : (gmax > g0 ? gmax - g0 : 0);
    if (ng <= 0 || ex.w2 == nullptr || ex.w1 == nullptr || ex.w3 == nullptr || ex.bits != BITS || ex.group != group ||
        ex.z1 != nullptr)
        return 0;
    const int nt = ng * TPG;
    gu4_t w2 = as_global<uint4>(ex.w2) + ((size_t)rb * tiles_k2 + (size_t)g0 * TPG) * 64 + lane;
    gu16_t s2 = as_global<uint16_t>(ex.s2) + (size_t)g0 * H + rb * 32 + n;
#pragma unroll
    for (int j = 0; j < kB1MaxTiles; ++j) raw[j] = w2[(size_t)(j < nt ? j : nt - 1) * 64];
#pragma unroll
    for (int jg = 0; jg < MAXG; ++jg) sc[jg] = s2[(size_t)(jg < ng ? jg : ng - 1) * H];
    return ng;
}

// Polls the h of the item's K range, then multiplies.  The codes enter the matrix cores as
// u + C (one v_and_or_b32 per pair); the constant's share, C + zero times the sum of the group's h,
// leaves per group - every lane holds one tagged word of a group of 128, so that sum is one wave
// reduction per group.  Returns the item's contribution to output row rb*32 + n in lanes 0..31.
template <int BITS, int TPG>
__device__ __forceinline__ float b1_down_product(const uint4 (&raw)[kB1MaxTiles], const uint32_t (&sc)[kB1MaxTiles / TPG],
                                                 int ng, const unsigned long long* hq_src, uint32_t tag, _Float16* hl,
                                                 const _Float16* zrow, bool* failed,
                                                 const unsigned long long* side = nullptr,
                                                 unsigned long long* side_val = nullptr) {
    constexpr int KT = QFmt<BITS>::KT, S = QFmt<BITS>::MSTEPS, MAXG = kB1MaxTiles / TPG;
    static_assert(KT * TPG == 128, "one tagged word of a group per lane");
    const int lane = threadIdx.x & 63;
    const int n = lane & 31, half = lane >> 5;
    float ch[MAXG];
    {
        const unsigned long long tagw = (unsigned long long)tag << 32;
        bool done = false;
        for (int it = 0; it < kSpinMax && !done; ++it) {
            unsigned long long v[MAXG];
#pragma unroll
            for (int j = 0; j < MAXG; ++j) v[j] = j < ng ? ld_dev(hq_src + lane + 64 * j) : tagw;
            // a word the caller needs right after the product rides along with every poll (side: this
            // lane's address or NULL), so that no memory round trip of its own follows the product
            if (side != nullptr) *side_val = ld_dev(side);
            bool good = true;
#pragma unroll
            for (int j = 0; j < MAXG; ++j) good = good && (uint32_t)(v[j] >> 32) == tag;
            if (__all(good)) {
                const float cc = BITS == 4 ? ((lane & 1) ? 72.f : 1032.f) : 1152.f;
#pragma unroll
                for (int j = 0; j < MAXG; ++j) {
                    const uint32_t w = (uint32_t)v[j];
                    reinterpret_cast<uint32_t*>(hl)[lane + 64 * j] = w;
                    const f16x2_t hv = __builtin_bit_cast(f16x2_t, w);
                    ch[j] = wave_sum(cc * ((float)hv.x + (float)hv.y));
                }
                done = true;
            } else {
                __builtin_amdgcn_s_sleep(2);
            }
        }
        if (!done) {
            *failed = true;
            return 0.f;
        }
    }
    const _Float16* ha = (n == 0 ? hl : zrow) + half * (KT / 2);
    const BiasConst bc = bias_const();
    const f32x16_t zero = f32x16_zero();
    float out = 0.f;
    // two groups at a time, each with an accumulator of its own: the dependent matrix-core steps
    // of one group run under those of the other
#pragma unroll
    for (int jg = 0; jg < MAXG; jg += 2) {
        constexpr bool kOdd = MAXG % 2 != 0;
        const bool pair = !kOdd || jg + 1 < MAXG;
        f32x16_t acc0, acc1 = zero;
#pragma unroll
        for (int tl = 0; tl < TPG; ++tl) {
            const int j0 = jg * TPG + tl, j1 = pair ? (jg + 1) * TPG + tl : j0;
            f16x8_t a0[S], a1[S], b0[S], b1[S];
#pragma unroll
            for (int st = 0; st < S; ++st) {
                a0[st] = *reinterpret_cast<const f16x8_t*>(ha + j0 * KT + 8 * st);
                if (pair) a1[st] = *reinterpret_cast<const f16x8_t*>(ha + j1 * KT + 8 * st);
            }
            biased_tile<BITS>(raw[j0], bc, b0);
            if (pair) biased_tile<BITS>(raw[j1], bc, b1);
#pragma unroll
            for (int st = 0; st < S; ++st) {
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0[st], b0[st], (tl == 0 && st == 0) ? zero : acc0, 0, 0, 0);
                if (pair)
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1[st], b1[st], (tl == 0 && st == 0) ? zero : acc1, 0, 0, 0);
            }
        }
        // groups past the item's end multiply stale h with repeated tiles: they do not count
        if (jg < ng) out = fmaf(half_bits_to_float(sc[jg]), acc0[0] - ch[jg], out);
        if (pair && jg + 1 < ng) out = fmaf(half_bits_to_float(sc[pair ? jg + 1 : jg]), acc1[0] - ch[pair ? jg + 1 : jg], out);
    }
    return out;
}

template <int BR, int TR, int BS, int TS>
__device__ __forceinline__ void b1_down_role(const B1Args& A, int part, int rb, uint32_t tag, char* dyn) {
    const LayerArgs& a = A.a;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int H = a.r.H, E = a.r.E, k = a.r.k;
    const B1DownLds L = b1_down_lds(E, k);
    _Float16* hl = reinterpret_cast<_Float16*>(dyn + L.hl) + wave * kB1HRegion;
    _Float16* zrow = reinterpret_cast<_Float16*>(dyn + L.zrow);
    float* red_s = reinterpret_cast<float*>(dyn + L.red);
    float* red_r = reinterpret_cast<float*>(dyn + L.red2);
    float* gate = reinterpret_cast<float*>(dyn + L.gate);
    uint4* tab = reinterpret_cast<uint4*>(dyn + L.tab);
    float* zl = reinterpret_cast<float*>(dyn + L.zl);
    int32_t* ids = reinterpret_cast<int32_t*>(dyn + L.ids);
    float* wv = reinterpret_cast<float*>(dyn + L.w);
    int32_t* src_e = reinterpret_cast<int32_t*>(dyn + L.src_e);
    int32_t* src_r = reinterpret_cast<int32_t*>(dyn + L.src_w);
    const B1Item its = A.items_s[part * kLayerWaves + wave], itr = A.items_r[part * kLayerWaves + wave];
    for (int c = tid; c < kB1HRegion / 8; c += kLayerThreads)
        *reinterpret_cast<uint4*>(zrow + c * 8) = make_uint4(0, 0, 0, 0);
    lds_barrier();
    bool failed = false;
    float out_s = 0.f, out_r = 0.f, wsrc = 1.f;

    // the wave's piece of a shared expert: requested at once
    uint4 raw_s[kB1MaxTiles];
    uint32_t sc_s[kB1MaxTiles / TS];
    int ng_s = 0;
    if (its.ng > 0) {
        const fate_qexpert ex = a.shared[its.src];
        ng_s = b1_down_request<BS, TS>(ex, H, rb, its.g0, its.ng, raw_s, sc_s);
    }
    const unsigned long long* hq_s = A.a.hq + (size_t)its.src * a.nkb_s * 16 + (size_t)its.g0 * 64;
    // the gate of the shared experts, evaluated behind those requests
    if (a.shared_gate != nullptr) {
        if (wave == 0) {
            const float g = wave_sigmoid_dot_bf16(reinterpret_cast<const uint4*>(a.r.x),
                                                  reinterpret_cast<const uint4*>(a.shared_gate), H >> 3);
            if (lane == 0) gate[0] = g;
        }
    } else if (tid == 0) {
        gate[0] = 1.f;
    }

    // the wave's piece of a routed slot: with a hint the hinted expert's W2 slice is requested before
    // the gate is known, else (or if the hint was wrong) as soon as the slot's expert is
    const int slot = itr.ng > 0 ? itr.src : 0;
    const unsigned long long* hq_r =
        A.a.hq + ((size_t)a.n_shared * a.nkb_s + (size_t)slot * a.nkb_r) * 16 + (size_t)itr.g0 * 64;
    uint4 raw_r[kB1MaxTiles];
    uint32_t sc_r[kB1MaxTiles / TR];
    // the block that writes y (two parts): its wave 0 reads the other part's partial output of its
    // row along with the polls of the routed h, lanes 0..31
    const unsigned long long* side = nullptr;
    unsigned long long side_val = 0;
    if (wave == 0 && lane < 32 && A.nparts == 2 && part == 1) side = A.a.yq + rb * 32 + lane;
    int e_cur = -1, ng_r = 0;
    if (a.hint != nullptr && itr.ng > 0) {
        e_cur = a.hint[slot];
        if (e_cur < 0 || e_cur >= E) e_cur = -1;
        if (e_cur >= 0) {
            const fate_qexpert exh = a.experts[e_cur];
            ng_r = b1_down_request<BR, TR>(exh, H, rb, itr.g0, itr.ng, raw_r, sc_r);
        }
    }
    int e_true = -1, rank = 0;
    if (!b1_slot_expert(A, tag, slot, tab, zl, ids, src_e, src_r, &e_true, &rank)) {
        failed = true;
    } else {
        if (itr.ng > 0 && e_true != e_cur) {
            ng_r = 0;
            if (e_true >= 0) {
                const fate_qexpert ex = reinterpret_cast<const fate_qexpert*>(tab)[e_true];
                ng_r = b1_down_request<BR, TR>(ex, H, rb, itr.g0, itr.ng, raw_r, sc_r);
            }
        }
        // the weights of the selection, while the requests are in flight
        if (wave == 0) wave_softmax_topk_rounds(zl, E, k, a.r.renorm, ids, wv);
        lds_barrier();
        wsrc = wv[rank];
    }
    // the shared piece first: its h exists long before the routed one
    if (ng_s > 0) out_s = b1_down_product<BS, TS>(raw_s, sc_s, ng_s, hq_s, tag, hl, zrow, &failed);
    if (ng_r > 0 && !failed)
        out_r = b1_down_product<BR, TR>(raw_r, sc_r, ng_r, hq_r, tag, hl, zrow, &failed, side, &side_val);
    if (failed && lane == 0) atomicOr(a.status, 2);
    if (lane < 32) {
        red_s[wave * 32 + lane] = out_s;
        red_r[wave * 32 + lane] = wsrc * out_r;
    }
    __syncthreads();
    if (tid < 32) {
        float v = gate[0] * ((red_s[tid] + red_s[32 + tid]) + (red_s[64 + tid] + red_s[96 + tid])) +
                  ((red_r[tid] + red_r[32 + tid]) + (red_r[64 + tid] + red_r[96 + tid]));
        const int row = rb * 32 + tid;
        if (part + 1 < A.nparts) {
            __hip_atomic_store(A.a.yq + (size_t)part * H + row,
                               ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(v),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            // the block that writes y: the other blocks' partial outputs, in block order, then its own
            float sum = 0.f;
            bool good = true;
            for (int p = 0; p + 1 < A.nparts; ++p) {
                const unsigned long long* src = A.a.yq + (size_t)p * H + row;
                unsigned long long w = side != nullptr ? side_val : 0;      // (two parts: p = 0 is the side word)
                int spin = 0;
                if (side != nullptr && (uint32_t)(w >> 32) == tag) {
                    sum += __uint_as_float((uint32_t)w);
                    continue;
                }
                for (; spin < kSpinMax; ++spin) {
                    w = ld_dev(src);
                    if ((uint32_t)(w >> 32) == tag) break;
                    __builtin_amdgcn_s_sleep(4);
                }
                good = good && spin < kSpinMax;
                sum += __uint_as_float((uint32_t)w);
            }
            if (!good) atomicOr(a.status, 2);
            v += sum;
            if (a.y_is_fp32) static_cast<float*>(a.y)[row] = v;
            else static_cast<uint16_t*>(a.y)[row] = (uint16_t)f32_to_bf16_bits(v);
        }
    }
}

template <int BR, int TR, int BS, int TS>
__global__ __launch_bounds__(kLayerThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void moe_layer_decode_b1_kernel(B1Args A) {
    extern __shared__ uint4 smem[];
    __shared__ FusedRouteSmem rsm;
    char* dyn = reinterpret_cast<char*>(smem);
    const LayerArgs& a = A.a;
    uint32_t tag = (uint32_t)ld_dev(a.sync) + 1u;
    if (tag == 0u) tag = 1u;
    int b = blockIdx.x;
    const int nd = A.nparts * A.nrb;
    if (b < a.nb_route) {
        route_role(a, b, tag, dyn, rsm);
    } else if ((b -= a.nb_route) < A.n_up_s) {
        b1_up_role<BR, TR, BS, TS, false>(A, b, true, tag, dyn);
    } else if ((b -= A.n_up_s) < A.n_up_r) {
        // (two copies of the routed up block: without a hint there is one place that asks for weights)
        if (a.hint != nullptr) b1_up_role<BR, TR, BS, TS, true>(A, b, false, tag, dyn);
        else b1_up_role<BR, TR, BS, TS, false>(A, b, false, tag, dyn);
    } else if ((b -= A.n_up_r) < nd) {
        b1_down_role<BR, TR, BS, TS>(A, b / A.nrb, b % A.nrb, tag, dyn);
    }
    // the workgroup that leaves last opens the next epoch
    __syncthreads();
    if (threadIdx.x == 0 && atomicAdd(a.sync + 1, 1) == (int)gridDim.x - 1) {
        st_dev(a.sync + 1, 0);
        st_dev(a.sync, (int32_t)tag);
    }
}

// ---- host side ----------------------------------------------------------------------------------
static bool b1_format(int bits, int group) { return (bits == 4 && group == 128) || (bits == 8 && group == 128); }

static int b1_lds_bytes(const fate_ffn_desc& d) {
    return std::max(work_lds(1, d.H, d.E, d.k).bytes, b1_down_lds(d.E, d.k).bytes);
}

template <int BR, int TR, int BS, int TS>
static int b1_occupancy(int lds) {
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(
            &nb, reinterpret_cast<const void*>(moe_layer_decode_b1_kernel<BR, TR, BS, TS>), kLayerThreads,
            (size_t)lds) != hipSuccess)
        return 0;
    return nb;
}

#define FATE_B1_SWITCH(bits_r, bits_s, BODY)          \
    if ((bits_r) == 4 && (bits_s) == 4) { BODY(4, 2, 4, 2) }      \
    else if ((bits_r) == 4) { BODY(4, 2, 8, 4) }                   \
    else if ((bits_s) == 4) { BODY(8, 4, 4, 2) }                   \
    else { BODY(8, 4, 8, 4) }

int b1_resident_blocks(const fate_ffn_desc& d) {
    static int cached_cu = 0;
    if (cached_cu == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cached_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return 0;
    }
    const int bits_s = d.n_shared ? d.shared_bits : d.bits;
    const int lds = b1_lds_bytes(d);
    // the occupancy query is not free: one answer per format pair and LDS size is kept
    static int key_lds[4] = {-1, -1, -1, -1}, val[4] = {0, 0, 0, 0};
    const int key = (d.bits == 8 ? 2 : 0) + (bits_s == 8 ? 1 : 0);
    if (key_lds[key] != lds) {
        int per_cu = 0;
#define FATE_B1_OCC(BR, TR, BS, TS) per_cu = b1_occupancy<BR, TR, BS, TS>(lds);
        FATE_B1_SWITCH(d.bits, bits_s, FATE_B1_OCC)
#undef FATE_B1_OCC
        val[key] = per_cu;
        key_lds[key] = lds;
    }
    return val[key] * cached_cu;
}

// Splits G groups of a source into wave items of at most maxg groups, as evenly as possible.
static int b1_add_items(B1Item* items, int n, int src, int G, int maxg) {
    const int pieces = (G + maxg - 1) / maxg;
    int g0 = 0;
    for (int p = 0; p < pieces; ++p) {
        const int ng = G / pieces + (p < G % pieces ? 1 : 0);
        if (n >= kB1MaxItems) return -1;
        items[n++] = B1Item{(int16_t)src, (int16_t)g0, (int16_t)ng, 0};
        g0 += ng;
    }
    return n;
}

bool b1_plan(const fate_ffn_desc& d, const LayerArgs& a, B1Args* b, int* nblocks) {
    if (d.N != 1 || d.k > kTokPass) return false;
    const int bits_s = d.n_shared ? d.shared_bits : d.bits, group_s = d.n_shared ? d.shared_group : d.group;
    if (!b1_format(d.bits, d.group) || !b1_format(bits_s, group_s)) return false;
    // the straight-line up projection: a whole number of register rings per wave
    const int kt_r = d.bits == 4 ? 64 : 32, kt_s = bits_s == 4 ? 64 : 32;
    if (d.H % (kLayerWaves * kUpRing * kt_r) || d.H % (kLayerWaves * kUpRing * kt_s)) return false;
    if (d.I_max % 128 || (d.n_shared && d.I_shared_max % 128)) return false;
    b->a = a;
    b->nrb = d.H / 32;
    b->n_up_s = d.n_shared * a.nkb_s;
    b->n_up_r = d.k * a.nkb_r;
    for (int i = 0; i < kB1MaxItems; ++i) b->items_s[i] = b->items_r[i] = B1Item{0, 0, 0, 0};
    int ns = 0, nr = 0;
    const int maxg_s = kB1MaxTiles / (group_s / kt_s), maxg_r = kB1MaxTiles / (d.group / kt_r);
    for (int s = 0; s < d.n_shared; ++s)
        if ((ns = b1_add_items(b->items_s, ns, s, d.I_shared_max / group_s, maxg_s)) < 0) return false;
    for (int j = 0; j < d.k; ++j)
        if ((nr = b1_add_items(b->items_r, nr, j, d.I_max / d.group, maxg_r)) < 0) return false;
    b->nparts = (std::max(ns, nr) + kLayerWaves - 1) / kLayerWaves;
    if (b->nparts < 1 || b->nparts > kLayerMaxParts) return false;
    *nblocks = a.nb_route + b->n_up_s + b->n_up_r + b->nparts * b->nrb;
    // The routing blocks and the shared experts' up blocks must be on the device from the start
    // (their requests do not wait for anything); the other blocks have nothing to do before the
    // logits exist and may start as earlier blocks leave (a block only waits for lower ids) - the
    // down blocks then ask for their shared W2 pieces later, nothing else changes.  A launch
    // several times larger than the device is left to the general kernel.
    const int resident = b1_resident_blocks(d);
    const int early = a.nb_route + b->n_up_s;
    return resident > 0 && early <= resident && *nblocks <= 2 * resident;
}

fate_status launch_layer_decode_b1(hipStream_t st, const fate_ffn_desc& d, const B1Args& b, int nblocks) {
    const int bits_s = d.n_shared ? d.shared_bits : d.bits;
    const int lds = b1_lds_bytes(d);
#define FATE_B1_LAUNCH(BR, TR, BS, TS) \
    moe_layer_decode_b1_kernel<BR, TR, BS, TS><<<nblocks, kLayerThreads, lds, st>>>(b);
    FATE_B1_SWITCH(d.bits, bits_s, FATE_B1_LAUNCH)
#undef FATE_B1_LAUNCH
    FATE_HIP(hipGetLastError());
    return FATE_OK;
}


}  // namespace fate
