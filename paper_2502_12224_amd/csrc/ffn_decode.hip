// Decode-side expert FFN: bandwidth-bound dequant-GEMV kernels.
//
// Two launches per layer.
//  up:   a workgroup owns 32 intermediate neurons of one activated expert (or
//        of a shared expert): it streams the matching 32-row blocks of W1 and
//        W3 (device-native 1 KiB tiles, one contiguous KiB per wave load),
//        the four waves splitting the reduction dimension, and writes
//        h = silu(W1 x) * (W3 x) as fp16.  It also clears its slice of y.
//  down: a workgroup owns 32 output rows of W2 of one expert and a chunk of
//        the reduction dimension, and adds weight * (W2 h) into y (fp32
//        atomics; at most a few contributions per element).
// Every wave requests its first D weight tiles before anything else and keeps
// D tiles per matrix in flight (register ring), so the HBM stream starts
// while the activations are still being staged in LDS.
// Codes are widened in registers (qformat.h); the per-group fp16 scale is
// applied to the fp32 group partial sum, so each weight enters exactly.
#include <hip/hip_fp16.h>
#include "common.h"
#include "qformat.h"
#include "ffn_internal.h"

namespace fate {

constexpr int kRingUp = 6;     // weight tiles in flight per matrix per wave (two matrices)
constexpr int kRingDown = 8;   // same for the single-matrix down kernel

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
__device__ __forceinline__ float half_bits_to_float(uint32_t b) { return __half2float(__ushort_as_half((unsigned short)b)); }

template <int NMAT, int D>
struct TileRing {
    uint4 raw[NMAT][D];
    uint32_t sc[NMAT][D];   // fp16 bits, one full register each (no 16-bit merges on arrival)
    int pf_g, pf_tl;   // group / position-in-group of the next tile to request
};

// request the first D tiles of [g_beg*tpg, g_end*tpg)
template <int NMAT, int D>
__device__ __forceinline__ void ring_start(TileRing<NMAT, D>& r, const gu4_t* wt, const gu16_t* sc,
                                           int g_beg, int g_end, int tpg) {
    const int tbeg = g_beg * tpg, tend = g_end * tpg;
    int g = g_beg, tl = 0;
#pragma unroll
    for (int j = 0; j < D; ++j) {
        if (tbeg + j < tend) {
#pragma unroll
            for (int i = 0; i < NMAT; ++i) {
                r.raw[i][j] = wt[i][(size_t)(tbeg + j) * 64];
                r.sc[i][j] = sc[i][g];
            }
        }
        if (++tl == tpg) { tl = 0; ++g; }
    }
    r.pf_g = g;
    r.pf_tl = tl;
}

// One wave accumulates, for up to TT activation rows held in LDS, the dot
// products of NMAT weight row-blocks (one row per lane pair) over the groups
// [g_beg, g_end); ring_start must have been called with the same range.
// xs: activations as dwords (pairs), row stride ldx_dw; xs16: per row, sums of
// each run of 16 activations; column 0 of both = absolute column k_base.
template <int BITS, bool F16, int TT, int NMAT, int D>
__device__ __forceinline__ void ring_run(TileRing<NMAT, D>& r, const gu4_t* wt, const gu16_t* sc,
                                         int g_beg, int g_end, int tpg, const uint32_t* xs, int ldx_dw,
                                         int k_base, const float* xs16, int ld16, int nt,
                                         float (&out)[NMAT][TT]) {
    constexpr int KT = QFmt<BITS>::KT, NP = QFmt<BITS>::NP;
    constexpr float OFF = q_offset<BITS, F16>();
    const int half = (threadIdx.x & 63) >> 5;
    const int tbeg = g_beg * tpg, tend = g_end * tpg;
    float ga[NMAT][TT], gx[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        gx[t] = 0.f;
#pragma unroll
        for (int i = 0; i < NMAT; ++i) ga[i][t] = 0.f;
    }
    int tl = 0;
    for (int base = tbeg; base < tend; base += D) {
#pragma unroll
        for (int j = 0; j < D; ++j) {
            const int tile = base + j;
            if (tile < tend) {
                uint32_t p[NMAT][NP];
                float s[NMAT];
#pragma unroll
                for (int i = 0; i < NMAT; ++i) {
                    unpack_pairs<BITS, F16>(r.raw[i][j], p[i]);
                    s[i] = half_bits_to_float(r.sc[i][j]);
                }
                if (tile + D < tend) {
#pragma unroll
                    for (int i = 0; i < NMAT; ++i) {
                        r.raw[i][j] = wt[i][(size_t)(tile + D) * 64];
                        r.sc[i][j] = sc[i][r.pf_g];
                    }
                }
                if (++r.pf_tl == tpg) { r.pf_tl = 0; ++r.pf_g; }
                const int kloc = tile * KT - k_base + half * (KT / 2);
#pragma unroll
                for (int t = 0; t < TT; ++t) {
                    if (t < nt) {
                        const uint4* xr = reinterpret_cast<const uint4*>(xs + t * ldx_dw + (kloc >> 1));
#pragma unroll
                        for (int q = 0; q < NP / 4; ++q) {
                            uint4 xv = xr[q];
#pragma unroll
                            for (int i = 0; i < NMAT; ++i) {
                                ga[i][t] = dot2<F16>(xv.x, p[i][4 * q + 0], ga[i][t]);
                                ga[i][t] = dot2<F16>(xv.y, p[i][4 * q + 1], ga[i][t]);
                                ga[i][t] = dot2<F16>(xv.z, p[i][4 * q + 2], ga[i][t]);
                                ga[i][t] = dot2<F16>(xv.w, p[i][4 * q + 3], ga[i][t]);
                            }
                        }
                        const float* px = xs16 + t * ld16 + (kloc >> 4);
                        if constexpr (BITS == 4) gx[t] += px[0] + px[1]; else gx[t] += px[0];
                    }
                }
                if (++tl == tpg) {
                    tl = 0;
#pragma unroll
                    for (int t = 0; t < TT; ++t) {
#pragma unroll
                        for (int i = 0; i < NMAT; ++i) {
                            out[i][t] = fmaf(s[i], fmaf(-OFF, gx[t], ga[i][t]), out[i][t]);
                            ga[i][t] = 0.f;
                        }
                        gx[t] = 0.f;
                    }
                }
            }
        }
    }
}

__device__ __forceinline__ float sum8_bf16(const uint4& v) {
    return ((bf16_lo(v.x) + bf16_hi(v.x)) + (bf16_lo(v.y) + bf16_hi(v.y))) +
           ((bf16_lo(v.z) + bf16_hi(v.z)) + (bf16_lo(v.w) + bf16_hi(v.w)));
}
__device__ __forceinline__ float sum8_f16(const uint4& v) {
    const __half2* h = reinterpret_cast<const __half2*>(&v);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) s += __low2float(h[i]) + __high2float(h[i]);
    return s;
}

template <int TT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void ffn_up_decode_kernel(DecodeArgs a) {
    extern __shared__ uint4 smem[];
    __shared__ float red[2][4][TT][32];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
#ifdef FATE_PROBE
    unsigned long long ts[8];
    ts[0] = wall_clock64();
#define FATE_TS(i) ts[i] = wall_clock64()
#else
#define FATE_TS(i)
#endif
    int b = blockIdx.x;
    const int nrout = a.nact * a.rb_r;
    const fate_qexpert* ex;
    int rb, T, sbeg = 0, bits, group, ldh;
    __half* hbuf;
    const bool is_shared = b >= nrout;
    bool live = true;
    if (!is_shared) {
        const int slot = b / a.rb_r;
        rb = b % a.rb_r;
        const int e = a.order[slot];
        T = a.counts[e];
        live = T > 0;
        ex = a.experts + e;
        sbeg = a.offsets[e];
        bits = a.bits_r; group = a.group_r;
        hbuf = a.h_r + (size_t)sbeg * a.ldh_r; ldh = a.ldh_r;
    } else {
        b -= nrout;
        const int s = b / a.rb_s;
        rb = b % a.rb_s;
        ex = a.shared + s;
        T = a.N;
        bits = a.bits_s; group = a.group_s;
        hbuf = a.h_s + (size_t)s * a.N * a.ldh_s; ldh = a.ldh_s;
    }
    gu4_t w1 = nullptr;
    gu4_t w3 = nullptr;
    if (live) {
        live = rb * 32 < ex->I;
        w1 = as_global<uint4>(ex->w1);
        w3 = as_global<uint4>(ex->w3);
        if (live && (w1 == nullptr || w3 == nullptr)) {
            if (tid == 0) atomicOr(a.status, 1);
            live = false;
        }
    }
    const int H = a.H, nvec = H >> 3, G = H / group, ld16 = H >> 4;
    const int KT = bits == 4 ? 64 : 32;
    const int tiles_k = H / KT, tpg = group / KT;
    const int n = lane & 31;
    gu4_t wt[2];
    gu16_t sc[2];
    const int g_beg = G * wave / 4, g_end = G * (wave + 1) / 4;
    TileRing<2, kRingUp> ring;
    if (live) {
        wt[0] = w1 + (size_t)rb * tiles_k * 64 + lane;
        wt[1] = w3 + (size_t)rb * tiles_k * 64 + lane;
        sc[0] = as_global<uint16_t>(ex->s1) + (size_t)(rb * 32 + n) * G;
        sc[1] = as_global<uint16_t>(ex->s3) + (size_t)(rb * 32 + n) * G;
        FATE_TS(1);
        ring_start<2, kRingUp>(ring, wt, sc, g_beg, g_end, tpg);
    }
    FATE_TS(2);
    {   // clear this block's slice of y
        const long long total = (long long)a.N * a.H;
        const long long per = (total + gridDim.x - 1) / gridDim.x;
        const long long b0 = (long long)blockIdx.x * per;
        const long long b1 = b0 + per < total ? b0 + per : total;
        for (long long i = b0 + tid; i < b1; i += 256) a.y[i] = 0.f;
    }
    if (!live) return;
    uint32_t* xs = reinterpret_cast<uint32_t*>(smem);
    float* xs16 = reinterpret_cast<float*>(smem + (size_t)TT * nvec);
    const uint4* xg = reinterpret_cast<const uint4*>(a.x);

    for (int t0 = 0; t0 < T; t0 += TT) {
        const int nt = min(TT, T - t0);
        if (t0 > 0) {
            __syncthreads();
            ring_start<2, kRingUp>(ring, wt, sc, g_beg, g_end, tpg);
        }
        for (int idx = tid; idx < nt * nvec; idx += 256) {
            const int t = idx / nvec, c = idx - t * nvec;
            const int tok = is_shared ? t0 + t : a.perm[sbeg + t0 + t] / a.k;
            const uint4 v = xg[(size_t)tok * nvec + c];
            smem[t * nvec + c] = v;
            float s = sum8_bf16(v);
            s += __shfl_xor(s, 1, 64);
            if (!(c & 1)) xs16[t * ld16 + (c >> 1)] = s;
        }
        __syncthreads();
        FATE_TS(3);
        float out[2][TT];
#pragma unroll
        for (int t = 0; t < TT; ++t) out[0][t] = out[1][t] = 0.f;
        if (bits == 4)
            ring_run<4, false, TT, 2, kRingUp>(ring, wt, sc, g_beg, g_end, tpg, xs, H >> 1, 0, xs16, ld16, nt, out);
        else
            ring_run<8, false, TT, 2, kRingUp>(ring, wt, sc, g_beg, g_end, tpg, xs, H >> 1, 0, xs16, ld16, nt, out);
        FATE_TS(4);
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            float v1 = out[0][t] + __shfl_xor(out[0][t], 32, 64);
            float v3 = out[1][t] + __shfl_xor(out[1][t], 32, 64);
            if (lane < 32) { red[0][wave][t][lane] = v1; red[1][wave][t][lane] = v3; }
        }
        __syncthreads();
        if (tid < 32 * nt) {
            const int t = tid >> 5, nn = tid & 31;
            const float a1 = red[0][0][t][nn] + red[0][1][t][nn] + red[0][2][t][nn] + red[0][3][t][nn];
            const float a3 = red[1][0][t][nn] + red[1][1][t][nn] + red[1][2][t][nn] + red[1][3][t][nn];
            const float hv = a1 / (1.0f + expf(-a1)) * a3;
            hbuf[(size_t)(t0 + t) * ldh + rb * 32 + nn] = __float2half(hv);
        }
#ifdef FATE_PROBE
        FATE_TS(5);
        if (tid == 0 && (blockIdx.x == 0 || blockIdx.x == nrout || blockIdx.x == gridDim.x - 1)) {
            unsigned long long* o = reinterpret_cast<unsigned long long*>(a.status) + 8 +
                                    (blockIdx.x == 0 ? 0 : blockIdx.x == nrout ? 8 : 16);
            for (int i = 0; i < 6; ++i) o[i] = ts[i];
        }
#endif
    }
}

template <int TT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void ffn_down_decode_kernel(DecodeArgs a) {
    extern __shared__ uint4 smem[];
    __shared__ float red[4][TT][32];
    __shared__ float sgate[TT];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nrb = a.H >> 5;
    int b = blockIdx.x;
    const int nrout = a.nact * nrb * a.nchunk_r;
    const fate_qexpert* ex;
    int rb, ch, cg, T, sbeg = 0, bits, group, ldh;
    const __half* hbuf;
    const bool is_shared = b >= nrout;
    if (!is_shared) {
        const int slot = b / (nrb * a.nchunk_r);
        const int rem = b - slot * (nrb * a.nchunk_r);
        rb = rem / a.nchunk_r; ch = rem - rb * a.nchunk_r; cg = a.cg_r;
        const int e = a.order[slot];
        T = a.counts[e];
        if (T == 0) return;
        ex = a.experts + e;
        sbeg = a.offsets[e];
        bits = a.bits_r; group = a.group_r;
        hbuf = a.h_r + (size_t)sbeg * a.ldh_r; ldh = a.ldh_r;
    } else {
        b -= nrout;
        const int s = b / (nrb * a.nchunk_s);
        const int rem = b - s * (nrb * a.nchunk_s);
        rb = rem / a.nchunk_s; ch = rem - rb * a.nchunk_s; cg = a.cg_s;
        ex = a.shared + s;
        T = a.N;
        bits = a.bits_s; group = a.group_s;
        hbuf = a.h_s + (size_t)s * a.N * a.ldh_s; ldh = a.ldh_s;
    }
    const int I = ex->I, G = I / group;
    const int gb = ch * cg, ge = min(G, gb + cg);
    if (gb >= ge) return;
    gu4_t w2 = as_global<uint4>(ex->w2);
    if (w2 == nullptr) return;   // flagged by the up kernel
    const int KT = bits == 4 ? 64 : 32;
    const int tiles_k = I / KT, tpg = group / KT;
    const int n = lane & 31;
    gu4_t wt[1] = {w2 + (size_t)rb * tiles_k * 64 + lane};
    gu16_t sc[1] = {as_global<uint16_t>(ex->s2) + (size_t)(rb * 32 + n) * G};
    const int ng = ge - gb;
    const int g_beg = gb + ng * wave / 4, g_end = gb + ng * (wave + 1) / 4;
    TileRing<1, kRingDown> ring;
    ring_start<1, kRingDown>(ring, wt, sc, g_beg, g_end, tpg);
    const int Kc = ng * group, kvec = Kc >> 3, k_base = gb * group, ld16 = Kc >> 4;
    uint32_t* xs = reinterpret_cast<uint32_t*>(smem);
    float* xs16 = reinterpret_cast<float*>(smem + (size_t)TT * kvec);

    for (int t0 = 0; t0 < T; t0 += TT) {
        const int nt = min(TT, T - t0);
        if (t0 > 0) {
            __syncthreads();
            ring_start<1, kRingDown>(ring, wt, sc, g_beg, g_end, tpg);
        }
        for (int idx = tid; idx < nt * kvec; idx += 256) {
            const int t = idx / kvec, c = idx - t * kvec;
            const uint4 v = *reinterpret_cast<const uint4*>(hbuf + (size_t)(t0 + t) * ldh + k_base + c * 8);
            smem[t * kvec + c] = v;
            float s = sum8_f16(v);
            s += __shfl_xor(s, 1, 64);
            if (!(c & 1)) xs16[t * ld16 + (c >> 1)] = s;
        }
        if (is_shared && a.shared_gate != nullptr) {
            const uint4* sgv = reinterpret_cast<const uint4*>(a.shared_gate);
            const int nvec = a.H >> 3;
            for (int t = wave; t < nt; t += 4) {
                const uint4* xr = reinterpret_cast<const uint4*>(a.x) + (size_t)(t0 + t) * nvec;
                float acc = 0.f;
                for (int c = lane; c < nvec; c += 64) {
                    uint4 xv = xr[c], gv = sgv[c];
                    acc = fmaf(bf16_lo(xv.x), bf16_lo(gv.x), acc); acc = fmaf(bf16_hi(xv.x), bf16_hi(gv.x), acc);
                    acc = fmaf(bf16_lo(xv.y), bf16_lo(gv.y), acc); acc = fmaf(bf16_hi(xv.y), bf16_hi(gv.y), acc);
                    acc = fmaf(bf16_lo(xv.z), bf16_lo(gv.z), acc); acc = fmaf(bf16_hi(xv.z), bf16_hi(gv.z), acc);
                    acc = fmaf(bf16_lo(xv.w), bf16_lo(gv.w), acc); acc = fmaf(bf16_hi(xv.w), bf16_hi(gv.w), acc);
                }
                acc = wave_sum(acc);
                if (lane == 0) sgate[t] = 1.0f / (1.0f + expf(-acc));
            }
        }
        __syncthreads();
        float out[1][TT];
#pragma unroll
        for (int t = 0; t < TT; ++t) out[0][t] = 0.f;
        if (bits == 4)
            ring_run<4, true, TT, 1, kRingDown>(ring, wt, sc, g_beg, g_end, tpg, xs, Kc >> 1, k_base, xs16, ld16, nt, out);
        else
            ring_run<8, true, TT, 1, kRingDown>(ring, wt, sc, g_beg, g_end, tpg, xs, Kc >> 1, k_base, xs16, ld16, nt, out);
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            float v = out[0][t] + __shfl_xor(out[0][t], 32, 64);
            if (lane < 32) red[wave][t][lane] = v;
        }
        __syncthreads();
        if (tid < 32 * nt) {
            const int t = tid >> 5, nn = tid & 31;
            const float v = red[0][t][nn] + red[1][t][nn] + red[2][t][nn] + red[3][t][nn];
            int tok;
            float wgt;
            if (is_shared) {
                tok = t0 + t;
                wgt = a.shared_gate ? sgate[t] : 1.0f;
            } else {
                const int p = a.perm[sbeg + t0 + t];
                tok = p / a.k;
                wgt = a.topk_w[p];
            }
            atomicAdd(a.y + (size_t)tok * a.H + rb * 32 + nn, wgt * v);
        }
    }
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ src, uint16_t* __restrict__ dst, long long n) {
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = (uint16_t)f32_to_bf16_bits(src[i]);
}

fate_status launch_ffn_decode(hipStream_t st, const fate_ffn_desc& d, DecodeArgs a, void* y_out) {
    int TT = d.N <= 1 ? 1 : d.N <= 2 ? 2 : d.N <= 4 ? 4 : 8;
    // LDS of the up kernel: TT rows of x (bf16) + their 16-wide sums; of the down kernel: TT rows of an h chunk
    auto lds_up = [&](int tt) { return (size_t)tt * d.H * 2 + (size_t)tt * (d.H / 16) * 4; };
    const int Gr = d.I_max / d.group, Gs = d.n_shared ? d.I_shared_max / d.shared_group : 0;
    a.nchunk_r = (Gr + 15) / 16; a.cg_r = (Gr + a.nchunk_r - 1) / a.nchunk_r;
    a.nchunk_s = Gs ? (Gs + 15) / 16 : 1; a.cg_s = Gs ? (Gs + a.nchunk_s - 1) / a.nchunk_s : 1;
    auto lds_down = [&](int tt) {
        size_t kr = (size_t)a.cg_r * d.group, ks = d.n_shared ? (size_t)a.cg_s * d.shared_group : 0;
        size_t kc = kr > ks ? kr : ks;
        return (size_t)tt * kc * 2 + (size_t)tt * (kc / 16) * 4;
    };
    while (TT > 1 && (lds_up(TT) > 40960 || lds_down(TT) > 40960)) TT >>= 1;
    if (lds_up(TT) > 40960 || lds_down(TT) > 40960)
        FATE_FAIL(FATE_ESHAPE, "H = %d too large for the decode kernels", d.H);
    a.nact = min(d.E, d.N * d.k);
    a.rb_r = d.I_max / 32;
    a.rb_s = d.n_shared ? d.I_shared_max / 32 : 0;
    const int grid_up = a.nact * a.rb_r + d.n_shared * a.rb_s;
    const int nrb = d.H / 32;
    const int grid_down = a.nact * nrb * a.nchunk_r + d.n_shared * nrb * a.nchunk_s;
    const size_t lu = lds_up(TT), ld = lds_down(TT);
    const bool do_up = d.phases != 2, do_down = d.phases != 1;
#define FATE_LAUNCH_DECODE(TTV)                                                   \
    if (do_up) ffn_up_decode_kernel<TTV><<<grid_up, 256, lu, st>>>(a);           \
    if (do_down) ffn_down_decode_kernel<TTV><<<grid_down, 256, ld, st>>>(a);
    switch (TT) {
        case 8: FATE_LAUNCH_DECODE(8) break;
        case 4: FATE_LAUNCH_DECODE(4) break;
        case 2: FATE_LAUNCH_DECODE(2) break;
        default: FATE_LAUNCH_DECODE(1) break;
    }
#undef FATE_LAUNCH_DECODE
    FATE_HIP(hipGetLastError());
    if (!d.y_is_fp32 && do_down) {
        const long long n = (long long)d.N * d.H;
        f32_to_bf16_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(a.y, static_cast<uint16_t*>(y_out), n);
        FATE_HIP(hipGetLastError());
    }
    return FATE_OK;
}

}  // namespace fate
