// Device-side building blocks of routing: wave-level softmax + top-m
// selection, and the stable token-to-expert permutation (one-wave form for
// up to 64 pairs, workgroup form for any number).
#pragma once
#include "common.h"

namespace fate {

constexpr int kVPL = kMaxE / 64;   // values per lane when a wave holds E <= 256 entries

__device__ __forceinline__ float lane_bcast(float v, int src) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src));
}
__device__ __forceinline__ int lane_bcast(int v, int src) { return __builtin_amdgcn_readlane(v, src); }

// One wavefront turns E logits (z, readable by every lane) into the softmax
// over all experts and the m largest entries, ordered by logit descending
// with ties to the lower id.  Selection is by rank: every entry counts the
// entries that precede it in that order (the wave broadcasts one entry at a
// time), and the entries of rank < m write themselves to position rank.
// NS = ceil(E/64) values per lane.  ids_out/w_out may point to global or LDS
// memory.  pop (optional) receives +1 per selected expert.  renorm != 0
// divides the m weights by their sum.
template <int NS>
__device__ __forceinline__ void wave_softmax_topm_ns(const float* z, int E, int m, int renorm,
                                                     int32_t* ids_out, float* w_out, float* probs_out,
                                                     int32_t* pop) {
    const int lane = threadIdx.x & 63;
    float v[NS];
    float lmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        int e = lane + 64 * i;
        float t = (e < E) ? z[e] : -INFINITY;
        if (t != t) t = -INFINITY;   // NaN logits are treated as -inf
        v[i] = t;
        lmax = fmaxf(lmax, t);
    }
    const float zmax = wave_max(lmax);
    float p[NS];
    float lsum = 0.f;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        p[i] = (lane + 64 * i < E) ? __expf(v[i] - zmax) : 0.f;
        lsum += p[i];
    }
    const float inv = 1.0f / wave_sum(lsum);
    int rank[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        p[i] *= inv;
        rank[i] = 0;
        if (probs_out && lane + 64 * i < E) probs_out[lane + 64 * i] = p[i];
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int lim = min(64, E - 64 * s);
        for (int src = 0; src < lim; ++src) {
            const float zj = lane_bcast(v[s], src);
            const int ej = src + 64 * s;
#pragma unroll
            for (int i = 0; i < NS; ++i) rank[i] += (zj > v[i]) || (zj == v[i] && ej < lane + 64 * i);
        }
    }
    float wsel = 0.f;
#pragma unroll
    for (int i = 0; i < NS; ++i)
        if (rank[i] < m && lane + 64 * i < E) wsel += p[i];
    const float scale = renorm ? 1.0f / wave_sum(wsel) : 1.0f;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int e = lane + 64 * i;
        if (e < E && rank[i] < m) {
            ids_out[rank[i]] = e;
            w_out[rank[i]] = p[i] * scale;
            if (pop) atomicAdd(&pop[e], 1);
        }
    }
}

__device__ __forceinline__ void wave_softmax_topm(const float* z, int E, int m, int renorm,
                                                  int32_t* ids_out, float* w_out, float* probs_out,
                                                  int32_t* pop) {
    if (E <= 64) wave_softmax_topm_ns<1>(z, E, m, renorm, ids_out, w_out, probs_out, pop);
    else if (E <= 128) wave_softmax_topm_ns<2>(z, E, m, renorm, ids_out, w_out, probs_out, pop);
    else wave_softmax_topm_ns<4>(z, E, m, renorm, ids_out, w_out, probs_out, pop);
}

// Stable grouping of P <= 64 pair indices by expert id, by ONE wavefront, in
// registers.  Same outputs as block_permute.  Every lane of the wave calls it.
template <int NS>
__device__ __forceinline__ void wave_permute_small_ns(const int32_t* ids, int P, int E, int32_t* counts,
                                                      int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                                                      int32_t* order) {
    const int lane = threadIdx.x & 63;
    const int ei = (lane < P) ? ids[lane] : -1;
    const bool valid = lane < P && ei >= 0 && ei < E;
    const int key = valid ? ei : -1;
    int cnt[NS], off[NS], rk[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) cnt[s] = rk[s] = 0;
    int before = 0;   // earlier pairs of the same expert
    for (int src = 0; src < P; ++src) {
        const int ej = lane_bcast(key, src);
        before += (ej == key) && (src < lane);
#pragma unroll
        for (int s = 0; s < NS; ++s) cnt[s] += (ej == lane + 64 * s);
    }
    int base = 0;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        // inclusive scan over the 64 lanes: DPP shifts inside rows of 16, then row carries
        int inc = cnt[s];
        inc += __builtin_amdgcn_update_dpp(0, inc, 0x111, 0xf, 0xf, true);   // row_shr:1
        inc += __builtin_amdgcn_update_dpp(0, inc, 0x112, 0xf, 0xf, true);   // row_shr:2
        inc += __builtin_amdgcn_update_dpp(0, inc, 0x114, 0xf, 0xf, true);   // row_shr:4
        inc += __builtin_amdgcn_update_dpp(0, inc, 0x118, 0xf, 0xf, true);   // row_shr:8
        const int r0 = lane_bcast(inc, 15), r1 = lane_bcast(inc, 31), r2 = lane_bcast(inc, 47),
                  r3 = lane_bcast(inc, 63);
        const int row = lane >> 4;
        inc += (row > 0 ? r0 : 0) + (row > 1 ? r1 : 0) + (row > 2 ? r2 : 0);
        off[s] = base + inc - cnt[s];
        base += r0 + r1 + r2 + r3;
        const int e = lane + 64 * s;
        if (e < E) {
            counts[e] = cnt[s];
            offsets[e] = off[s];
        }
    }
    if (lane == 0) offsets[E] = base;
    int myoff = 0;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        int t = __shfl(off[s], ei & 63, 64);
        if (valid && (ei >> 6) == s) myoff = t;
    }
    if (valid) {
        perm[myoff + before] = lane;
        inv_perm[lane] = myoff + before;
    } else if (lane < P) {
        inv_perm[lane] = -1;
    }
#pragma unroll
    for (int s2 = 0; s2 < NS; ++s2) {
        const int lim = min(64, E - 64 * s2);
        for (int src = 0; src < lim; ++src) {
            const int cj = lane_bcast(cnt[s2], src);
            const int ej = src + 64 * s2;
#pragma unroll
            for (int s = 0; s < NS; ++s) rk[s] += (cj > cnt[s]) || (cj == cnt[s] && ej < lane + 64 * s);
        }
    }
#pragma unroll
    for (int s = 0; s < NS; ++s)
        if (lane + 64 * s < E) order[rk[s]] = lane + 64 * s;
}

__device__ __forceinline__ void wave_permute_small(const int32_t* ids, int P, int E, int32_t* counts,
                                                   int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                                                   int32_t* order) {
    if (E <= 64) wave_permute_small_ns<1>(ids, P, E, counts, offsets, perm, inv_perm, order);
    else if (E <= 128) wave_permute_small_ns<2>(ids, P, E, counts, offsets, perm, inv_perm, order);
    else wave_permute_small_ns<4>(ids, P, E, counts, offsets, perm, inv_perm, order);
}

// The m largest of E logits by m rounds of arg-max: same ids, order and
// weights as wave_softmax_topm, cheaper when m is a handful (no loop over E).
template <int NS>
__device__ __forceinline__ void wave_softmax_topk_rounds_ns(const float* z, int E, int m, int renorm,
                                                            int32_t* ids_out, float* w_out) {
    const int lane = threadIdx.x & 63;
    float v[NS];
    float lmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int e = lane + 64 * i;
        float t = (e < E) ? z[e] : -INFINITY;
        if (t != t) t = -INFINITY;
        v[i] = t;
        lmax = fmaxf(lmax, t);
    }
    const float zmax = wave_max(lmax);
    float p[NS];
    float lsum = 0.f;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        p[i] = (lane + 64 * i < E) ? __expf(v[i] - zmax) : 0.f;
        lsum += p[i];
    }
    const float inv = 1.0f / wave_sum(lsum);
    int myrank[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        p[i] *= inv;
        myrank[i] = -1;
    }
    for (int r = 0; r < m; ++r) {
        float lbest = -INFINITY;
#pragma unroll
        for (int i = 0; i < NS; ++i)
            if (lane + 64 * i < E && myrank[i] < 0) lbest = fmaxf(lbest, v[i]);
        const float vbest = wave_max(lbest);
        int found = -1;
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const unsigned long long ball = __ballot(lane + 64 * i < E && myrank[i] < 0 && v[i] == vbest);
            if (found < 0 && ball) found = 64 * i + __ffsll((long long)ball) - 1;
        }
#pragma unroll
        for (int i = 0; i < NS; ++i)
            if (found == lane + 64 * i) myrank[i] = r;
    }
    float wsel = 0.f;
#pragma unroll
    for (int i = 0; i < NS; ++i)
        if (myrank[i] >= 0) wsel += p[i];
    const float scale = renorm ? 1.0f / wave_sum(wsel) : 1.0f;
#pragma unroll
    for (int i = 0; i < NS; ++i)
        if (myrank[i] >= 0) {
            ids_out[myrank[i]] = lane + 64 * i;
            w_out[myrank[i]] = p[i] * scale;
        }
}

// The expert that wave_softmax_topk_rounds puts at rank r (0 = largest logit): its first r + 1
// rounds of arg-max and nothing else - no softmax, no weights - for a consumer that only has
// to know where to fetch from.  The result is the same in every lane.
template <int NS>
__device__ __forceinline__ int wave_rank_expert_ns(const float* z, int E, int r) {
    const int lane = threadIdx.x & 63;
    float v[NS];
    bool taken[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int e = lane + 64 * i;
        float t = (e < E) ? z[e] : -INFINITY;
        if (t != t) t = -INFINITY;
        v[i] = t;
        taken[i] = false;
    }
    int found = -1;
    for (int q = 0; q <= r; ++q) {
        float lbest = -INFINITY;
#pragma unroll
        for (int i = 0; i < NS; ++i)
            if (lane + 64 * i < E && !taken[i]) lbest = fmaxf(lbest, v[i]);
        const float vbest = wave_max(lbest);
        found = -1;
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const unsigned long long ball = __ballot(lane + 64 * i < E && !taken[i] && v[i] == vbest);
            if (found < 0 && ball) found = 64 * i + __ffsll((long long)ball) - 1;
        }
#pragma unroll
        for (int i = 0; i < NS; ++i)
            if (found == lane + 64 * i) taken[i] = true;
    }
    return found;
}
// The same rounds for all of the first m ranks: ids_out[r] = the expert of rank r (one wave).
template <int NS>
__device__ __forceinline__ void wave_topk_ids_ns(const float* z, int E, int m, int32_t* ids_out) {
    const int lane = threadIdx.x & 63;
    float v[NS];
    bool taken[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int e = lane + 64 * i;
        float t = (e < E) ? z[e] : -INFINITY;
        if (t != t) t = -INFINITY;
        v[i] = t;
        taken[i] = false;
    }
    for (int r = 0; r < m; ++r) {
        float lbest = -INFINITY;
#pragma unroll
        for (int i = 0; i < NS; ++i)
            if (lane + 64 * i < E && !taken[i]) lbest = fmaxf(lbest, v[i]);
        const float vbest = wave_max(lbest);
        int found = -1;
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const unsigned long long ball = __ballot(lane + 64 * i < E && !taken[i] && v[i] == vbest);
            if (found < 0 && ball) found = 64 * i + __ffsll((long long)ball) - 1;
        }
#pragma unroll
        for (int i = 0; i < NS; ++i)
            if (found == lane + 64 * i) taken[i] = true;
        if (lane == 0) ids_out[r] = found;
    }
}
__device__ __forceinline__ void wave_topk_ids(const float* z, int E, int m, int32_t* ids_out) {
    if (E <= 64) wave_topk_ids_ns<1>(z, E, m, ids_out);
    else if (E <= 128) wave_topk_ids_ns<2>(z, E, m, ids_out);
    else wave_topk_ids_ns<4>(z, E, m, ids_out);
}
__device__ __forceinline__ int wave_rank_expert(const float* z, int E, int r) {
    if (E <= 64) return wave_rank_expert_ns<1>(z, E, r);
    if (E <= 128) return wave_rank_expert_ns<2>(z, E, r);
    return wave_rank_expert_ns<4>(z, E, r);
}

__device__ __forceinline__ void wave_softmax_topk_rounds(const float* z, int E, int m, int renorm,
                                                         int32_t* ids_out, float* w_out) {
    if (E <= 64) wave_softmax_topk_rounds_ns<1>(z, E, m, renorm, ids_out, w_out);
    else if (E <= 128) wave_softmax_topk_rounds_ns<2>(z, E, m, renorm, ids_out, w_out);
    else wave_softmax_topk_rounds_ns<4>(z, E, m, renorm, ids_out, w_out);
}

// One wavefront, P <= 64 (token, expert) pairs in ids[]: the expert at position
// `slot` of the order (pair count descending, id ascending) - what
// expert_order[slot] of the permutation holds for an activated expert - or -1
// when fewer experts are activated.  *T_out = its pair count; a lane whose pair
// belongs to it gets *pos_out = the pair's position among them (pair order),
// other lanes -1.  The result is the same in every lane.
__device__ __forceinline__ int wave_slot_expert(const int32_t* ids, int P, int E, int slot, int* T_out,
                                                int* pos_out) {
    const int lane = threadIdx.x & 63;
    const int ei = (lane < P) ? ids[lane] : -1;
    const bool valid = lane < P && ei >= 0 && ei < E;
    const int key = valid ? ei : -1;
    int cnt = 0, before = 0;
    for (int src = 0; src < P; ++src) {
        const int ej = lane_bcast(key, src);
        const bool same = valid && ej == key;
        cnt += same;
        before += same && src < lane;
    }
    const int first = valid && before == 0;
    int rank = 0;
    for (int src = 0; src < P; ++src) {
        const int cj = lane_bcast(cnt, src), ej = lane_bcast(key, src), fj = lane_bcast(first, src);
        rank += fj && ((cj > cnt) || (cj == cnt && ej < key));
    }
    const unsigned long long ball = __ballot(first && rank == slot);
    *T_out = 0;
    *pos_out = -1;
    if (!ball) return -1;
    const int L = __ffsll((long long)ball) - 1;
    const int e = lane_bcast(key, L);
    *T_out = lane_bcast(cnt, L);
    if (valid && key == e) *pos_out = before;
    return e;
}

// One wavefront, P <= 64 pairs: what wave_slot_expert gives for one slot, for every slot at once.
// tab: [64 slots][2 + 3 * rows_max] words: expert (-1 past the activated ones), its pair count,
// then the tokens, pair indices and weights (float bits) of its pairs in pair order.  The caller
// has set every expert word to -1.  w: the pairs' routing weights.
__device__ __forceinline__ void wave_slot_table(const int32_t* ids, const float* w, int P, int E, int k_magic_div,
                                                uint32_t k_magic, int rows_max, int32_t* tab) {
    const int lane = threadIdx.x & 63;
    const int words = 2 + 3 * rows_max;
    const int ei = (lane < P) ? ids[lane] : -1;
    const bool valid = lane < P && ei >= 0 && ei < E;
    const int key = valid ? ei : -1;
    int cnt = 0, before = 0;
    for (int src = 0; src < P; ++src) {
        const int ej = lane_bcast(key, src);
        const bool same = valid && ej == key;
        cnt += same;
        before += same && src < lane;
    }
    const int first = valid && before == 0;
    int rank = 0;          // experts in front of this lane's expert in the order (pair count descending, id ascending)
    for (int src = 0; src < P; ++src) {
        const int cj = lane_bcast(cnt, src), ej = lane_bcast(key, src), fj = lane_bcast(first, src);
        rank += fj && ((cj > cnt) || (cj == cnt && ej < key));
    }
    if (valid && before < rows_max) {
        int32_t* t = tab + rank * words;
        if (first) { t[0] = key; t[1] = cnt; }
        t[2 + before] = k_magic ? (int)__umulhi((uint32_t)lane, k_magic) : lane / k_magic_div;
        t[2 + rows_max + before] = lane;
        t[2 + 2 * rows_max + before] = __float_as_int(w[lane]);
    }
}

// Per-lane mask of the lanes in this wave that hold the same key (valid lanes only).
__device__ __forceinline__ unsigned long long wave_match(int key, bool valid, int nbits) {
    unsigned long long mask = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
        bool bit = (key >> b) & 1;
        unsigned long long bb = __ballot(valid && bit);
        mask &= bit ? bb : ~bb;
    }
    return mask;
}

constexpr int kPermMaxWaves = 16;
constexpr int kPermSmemInts = (kPermMaxWaves + 2) * kMaxE;

// Stable grouping of P pair indices by expert id, by one workgroup of
// blockDim.x = 64*nw threads (nw <= 16).  sm: kPermSmemInts ints of LDS.
// Every thread of the block must call it.
__device__ inline void block_permute(const int32_t* ids, int P, int E, int32_t* counts, int32_t* offsets,
                                     int32_t* perm, int32_t* inv_perm, int32_t* order, volatile int32_t* sm) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nthreads = blockDim.x, nw = nthreads >> 6;
    volatile int32_t* wc = sm;                 // [nw][E] per-wave counts, then running bases
    volatile int32_t* tot = sm + nw * E;       // [E] totals
    volatile int32_t* excl = tot + E;          // [E] exclusive offsets
    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;
    int chunk = (P + nw - 1) / nw;
    chunk = (chunk + 63) & ~63;
    const int beg = wave * chunk;
    const int end = min(P, beg + chunk);
    const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));

    // the wave's first kPermCache * 64 ids stay in registers for both passes, requested at once
    constexpr int kPermCache = 8;
    int ec[kPermCache];
#pragma unroll
    for (int it = 0; it < kPermCache; ++it) {
        const int i = beg + 64 * it + lane;
        ec[it] = (i < end) ? ids[i] : -1;
    }
    for (int i = tid; i < nw * E; i += nthreads) wc[i] = 0;
    __syncthreads();
    auto count_step = [&](int base, int e) {
        int i = base + lane;
        bool valid = (i < end) && e >= 0 && e < E;
        unsigned long long mk = wave_match(e, valid, nbits);
        if (valid && (mk & lt) == 0) wc[wave * E + e] += __popcll(mk);
    };
#pragma unroll
    for (int it = 0; it < kPermCache; ++it)
        if (beg + 64 * it < end) count_step(beg + 64 * it, ec[it]);
    for (int base = beg + 64 * kPermCache; base < end; base += 64) {
        int i = base + lane;
        count_step(base, (i < end) ? ids[i] : -1);
    }
    __syncthreads();
    for (int e = tid; e < E; e += nthreads) {
        int run = 0;
        for (int w = 0; w < nw; ++w) {
            int c = wc[w * E + e];
            wc[w * E + e] = run;
            run += c;
        }
        tot[e] = run;
    }
    __syncthreads();
    if (wave == 0) {
        // exclusive scan over E <= 256 totals: 4 consecutive experts per lane
        int c[4], s = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int e = lane * 4 + i;
            c[i] = (e < E) ? tot[e] : 0;
            s += c[i];
        }
        int inc = s;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            int up = __shfl_up(inc, o, 64);
            if (lane >= o) inc += up;
        }
        int run = inc - s;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int e = lane * 4 + i;
            if (e < E) {
                excl[e] = run;
                counts[e] = c[i];
                offsets[e] = run;
            }
            run += c[i];
        }
        if (lane == 63) offsets[E] = inc;
    }
    __syncthreads();
    auto place_step = [&](int base, int e) {
        int i = base + lane;
        bool valid = (i < end) && e >= 0 && e < E;
        unsigned long long mk = wave_match(e, valid, nbits);
        int b = valid ? wc[wave * E + e] : 0;
        if (valid) {
            int pos = excl[e] + b + __popcll(mk & lt);
            perm[pos] = i;
            inv_perm[i] = pos;
        } else if (i < end) {
            inv_perm[i] = -1;
        }
        if (valid && (mk & lt) == 0) wc[wave * E + e] = b + __popcll(mk);
    };
#pragma unroll
    for (int it = 0; it < kPermCache; ++it)
        if (beg + 64 * it < end) place_step(beg + 64 * it, ec[it]);
    for (int base = beg + 64 * kPermCache; base < end; base += 64) {
        int i = base + lane;
        place_step(base, (i < end) ? ids[i] : -1);
    }
    // experts by (count descending, id ascending): lane o holds the totals of experts o, o + 64,
    // ..; an expert's rank is the number of experts that come before it, counted by ballots
    int cl[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) cl[g] = (lane + 64 * g < E) ? tot[lane + 64 * g] : -1;
    for (int e = wave; e < E; e += nw) {
        const int c = tot[e];
        int r = 0;
#pragma unroll
        for (int g = 0; g < 4; ++g)
            r += __popcll(__ballot(cl[g] > c || (cl[g] == c && lane + 64 * g < e)));
        if (lane == 0) order[r] = e;
    }
}

__device__ __forceinline__ float dot8_bf16(const uint4& a, const uint4& b, float acc) {
    acc = fmaf(bf16_lo(a.x), bf16_lo(b.x), acc);
    acc = fmaf(bf16_hi(a.x), bf16_hi(b.x), acc);
    acc = fmaf(bf16_lo(a.y), bf16_lo(b.y), acc);
    acc = fmaf(bf16_hi(a.y), bf16_hi(b.y), acc);
    acc = fmaf(bf16_lo(a.z), bf16_lo(b.z), acc);
    acc = fmaf(bf16_hi(a.z), bf16_hi(b.z), acc);
    acc = fmaf(bf16_lo(a.w), bf16_lo(b.w), acc);
    acc = fmaf(bf16_hi(a.w), bf16_hi(b.w), acc);
    return acc;
}

// ---- decode-side routing spread over workgroups ------------------------------
constexpr int kFusedMaxN = 16;

struct FusedRouteArgs {
    const uint16_t* x; const uint16_t* Wg; const float* bias;
    const uint16_t* Wg2; const float* bias2;      // next layer's gate (NULL: no prediction)
    int N, H, E, k, m, renorm;
    int32_t* ids; float* w; int32_t* pids; float* pw; int32_t* pop;
    int32_t* counts; int32_t* offsets; int32_t* perm; int32_t* inv_perm; int32_t* order;
    float* zbuf;                                  // [2][N][E] logits
};

struct FusedRouteSmem {
    float z[8][kMaxE];                            // one row per wave of the workgroup (at most 8)
    int32_t ids[kFusedMaxN * kMaxM];
    int32_t pop[kMaxE];
};

// Logits go through device-scope stores / loads: the selecting workgroup may
// sit on another compute die than the one that produced a logit.
struct ZbufStore {
    float* zbuf; int N, E;
    __device__ __forceinline__ void operator()(int g, int t, int e, float v) const {
        st_dev(zbuf + ((size_t)g * N + t) * E + e, v);
    }
};
struct ZbufLoad {
    const float* zbuf; int N, E;
    __device__ __forceinline__ float operator()(int g, int t, int e) const {
        return ld_dev(zbuf + ((size_t)g * N + t) * E + e);
    }
};

// Workgroup `rblock` of ceil(rows / waves-per-workgroup): each of its waves
// takes one gate row (of this layer's gate, then of the next layer's) against
// every token and hands each logit to store(g, token, expert, value).
template <class Store>
__device__ __forceinline__ void fused_gate_rows(const FusedRouteArgs& a, int rblock, const Store& store) {
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int N = a.N, E = a.E, nvec = a.H >> 3;
    const int nrows = a.Wg2 ? 2 * E : E;
    const uint4* xg = reinterpret_cast<const uint4*>(a.x);
    const int r = rblock * (int)(blockDim.x >> 6) + wave;
    if (r >= nrows) return;
    const int g = r >= E, e = g ? r - E : r;
    const uint4* wr = reinterpret_cast<const uint4*>(g ? a.Wg2 : a.Wg) + (size_t)e * nvec;
    const float* bb = g ? a.bias2 : a.bias;
    const float b = bb ? bb[e] : 0.f;
    for (int t0 = 0; t0 < N; t0 += 4) {
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int c0 = lane; c0 < nvec; c0 += 64 * 8) {
            // all requests of the batch go out before the first use
            uint4 wv[8], xv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = c0 + 64 * j;
                wv[j] = c < nvec ? wr[c] : make_uint4(0, 0, 0, 0);
                xv[j] = c < nvec ? xg[(size_t)t0 * nvec + c] : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int c = c0 + 64 * j;
                acc[0] = dot8_bf16(xv[j], wv[j], acc[0]);
                if (c < nvec) {
#pragma unroll
                    for (int t = 1; t < 4; ++t)
                        if (t0 + t < N) acc[t] = dot8_bf16(xg[(size_t)(t0 + t) * nvec + c], wv[j], acc[t]);
                }
            }
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            float s = wave_sum(acc[t]);
            if (lane == 0 && t0 + t < N) store(g, t0 + t, e, s + b);
        }
    }
}

// Run by one whole workgroup (4..8 waves) once every logit has been stored:
// softmax and selection per token, predicted popularity, permutation.
// load(g, token, expert) returns a logit.  sm_perm: kPermSmemInts ints, only
// touched when N*k > 64 (may be NULL otherwise).
template <class Load>
__device__ __forceinline__ void fused_select(const FusedRouteArgs& a, FusedRouteSmem& sm, int32_t* sm_perm,
                                             const Load& load) {
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nthreads = blockDim.x, nw = nthreads >> 6;
    const int N = a.N, E = a.E, k = a.k, m = a.m;
    for (int i = threadIdx.x; i < E; i += nthreads) sm.pop[i] = 0;
    __syncthreads();
    const int njobs = (a.Wg2 ? 2 : 1) * N;
    for (int j0 = 0; j0 < njobs; j0 += nw) {
        const int job = j0 + wave;
        const int g = job >= N, t = g ? job - N : job;
        if (job < njobs) {
            for (int e = lane; e < E; e += 64) sm.z[wave][e] = load(g, t, e);
            __builtin_amdgcn_wave_barrier();
            if (!g) {
                wave_softmax_topm(sm.z[wave], E, k, a.renorm, sm.ids + t * k, a.w + (size_t)t * k, nullptr, nullptr);
            } else {
                wave_softmax_topm(sm.z[wave], E, m, 0, a.pids + (size_t)t * m, a.pw + (size_t)t * m, nullptr, sm.pop);
            }
        }
    }
    __syncthreads();
    const int P = N * k;
    for (int i = threadIdx.x; i < P; i += nthreads) a.ids[i] = sm.ids[i];
    if (a.Wg2)
        for (int i = threadIdx.x; i < E; i += nthreads) a.pop[i] = sm.pop[i];
    if (P <= 64) {
        if (wave == 0) wave_permute_small(sm.ids, P, E, a.counts, a.offsets, a.perm, a.inv_perm, a.order);
    } else {
        block_permute(sm.ids, P, E, a.counts, a.offsets, a.perm, a.inv_perm, a.order, sm_perm);
    }
}

}  // namespace fate
