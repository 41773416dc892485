// Device-side building blocks of routing: wave-level softmax + top-m
// selection, and the block-level stable token-to-expert permutation.
#pragma once
#include "common.h"

namespace fate {

// One wavefront turns E logits (z, readable by every lane) into the softmax
// over all experts and the m largest entries, ordered by logit descending
// with ties to the lower id.  Lane j < m ends up with the j-th selection.
// ids_out/w_out may point to global or LDS memory.  pop (optional) receives
// +1 per selected expert.  renorm != 0 divides the m weights by their sum.
__device__ __forceinline__ void wave_softmax_topm(const float* z, int E, int m, int renorm,
                                                  int32_t* ids_out, float* w_out, float* probs_out,
                                                  int32_t* pop) {
    const int lane = threadIdx.x & 63;
    constexpr int VPL = kMaxE / 64;
    float v[VPL];
    float lmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        int e = lane + 64 * i;
        float t = (e < E) ? z[e] : -INFINITY;
        if (t != t) t = -INFINITY;   // NaN logits are treated as -inf
        v[i] = t;
        lmax = fmaxf(lmax, t);
    }
    const float zmax = wave_max(lmax);
    float lsum = 0.f;
#pragma unroll
    for (int i = 0; i < VPL; ++i) lsum += (lane + 64 * i < E) ? expf(v[i] - zmax) : 0.f;
    const float inv = 1.0f / wave_sum(lsum);
    if (probs_out) {
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            int e = lane + 64 * i;
            if (e < E) probs_out[e] = expf(v[i] - zmax) * inv;
        }
    }
    unsigned taken = 0;
    int my_id = 0;
    float my_w = 0.f;
    float wsum = 0.f;
    for (int j = 0; j < m; ++j) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            int e = lane + 64 * i;
            bool ok = (e < E) && !((taken >> i) & 1u);
            if (ok && (bi == 0x7fffffff || v[i] > bv)) { bv = v[i]; bi = e; }
        }
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) {
            float ov = __shfl_xor(bv, o, 64);
            int oi = __shfl_xor(bi, o, 64);
            if (oi != 0x7fffffff && (bi == 0x7fffffff || ov > bv || (ov == bv && oi < bi))) { bv = ov; bi = oi; }
        }
        if ((bi & 63) == lane) taken |= 1u << (bi >> 6);
        float wj = expf(bv - zmax) * inv;
        wsum += wj;
        if (lane == j) { my_id = bi; my_w = wj; }
    }
    if (renorm) my_w = my_w / wsum;
    if (lane < m) {
        ids_out[lane] = my_id;
        w_out[lane] = my_w;
        if (pop) atomicAdd(&pop[my_id], 1);
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
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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

    for (int i = tid; i < nw * E; i += nthreads) wc[i] = 0;
    __syncthreads();
    for (int base = beg; base < end; base += 64) {
        int i = base + lane;
        int e = (i < end) ? ids[i] : -1;
        bool valid = (i < end) && e >= 0 && e < E;
        unsigned long long mk = wave_match(e, valid, nbits);
        if (valid && (mk & lt) == 0) wc[wave * E + e] += __popcll(mk);
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
    for (int base = beg; base < end; base += 64) {
        int i = base + lane;
        int e = (i < end) ? ids[i] : -1;
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
    }
    for (int e = tid; e < E; e += nthreads) {
        int c = tot[e], r = 0;
        for (int o = 0; o < E; ++o) {
            int co = tot[o];
            r += (co > c) || (co == c && o < e);
        }
        order[r] = e;
    }
}

}  // namespace fate
