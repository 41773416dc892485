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
// Codes are widened in registers (qformat.h); the per-group fp16 scale is
// applied to the fp32 group partial sum, so each weight enters exactly.
#include <hip/hip_fp16.h>
#include "common.h"
#include "qformat.h"
#include "ffn_internal.h"

namespace fate {

// One wave accumulates, for up to TT activation rows held in LDS, the dot
// products of NMAT weight row-blocks (one row per lane pair) over the groups
// [g_beg, g_end).  wt[i]: tile pointer of the row-block, already offset by the
// lane; sc[i]: scale row of this lane's weight row.  xs: activations as
// dwords (pairs), row stride ldx_dw, column 0 of xs = absolute column k_base.
// xgs[(t*G + g)*2 + half]: sum of the activations this lane half multiplies
// in group g (absolute group index minus g_base).
template <int BITS, bool F16, int TT, int NMAT>
__device__ __forceinline__ void gemv_rowblock(const uint4* const* wt, const __half* const* sc, int g_beg,
                                              int g_end, int tpg, const uint32_t* xs, int ldx_dw, int k_base,
                                              const float* xgs, int G, int g_base, int nt,
                                              float (&out)[NMAT][TT]) {
    constexpr int KT = QFmt<BITS>::KT, NP = QFmt<BITS>::NP;
    constexpr float OFF = q_offset<BITS, F16>();
    const int half = (threadIdx.x & 63) >> 5;
    int tile = g_beg * tpg;
    const int tend = g_end * tpg;
    uint4 nxt[NMAT];
#pragma unroll
    for (int i = 0; i < NMAT; ++i) nxt[i] = (tile < tend) ? wt[i][(size_t)tile * 64] : make_uint4(0, 0, 0, 0);
    for (int g = g_beg; g < g_end; ++g) {
        float ga[NMAT][TT];
        float sg[NMAT];
#pragma unroll
        for (int i = 0; i < NMAT; ++i) {
            sg[i] = __half2float(sc[i][g]);
#pragma unroll
            for (int t = 0; t < TT; ++t) ga[i][t] = 0.f;
        }
        for (int tl = 0; tl < tpg; ++tl, ++tile) {
            uint32_t p[NMAT][NP];
#pragma unroll
            for (int i = 0; i < NMAT; ++i) {
                uint4 raw = nxt[i];
                if (tile + 1 < tend) nxt[i] = wt[i][(size_t)(tile + 1) * 64];
                unpack_pairs<BITS, F16>(raw, p[i]);
            }
            const int xoff = (tile * KT - k_base + half * (KT / 2)) >> 1;
#pragma unroll
            for (int t = 0; t < TT; ++t) {
                if (t < nt) {
                    const uint4* xr = reinterpret_cast<const uint4*>(xs + t * ldx_dw + xoff);
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
                }
            }
        }
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            if (t < nt) {
                float xsum = xgs[(t * G + (g - g_base)) * 2 + half];
#pragma unroll
                for (int i = 0; i < NMAT; ++i) out[i][t] = fmaf(sg[i], fmaf(-OFF, xsum, ga[i][t]), out[i][t]);
            }
        }
    }
}

// sums of 16-bit activations over the column segments a lane half multiplies
template <bool F16>
__device__ __forceinline__ void group_half_sums(const uint32_t* xs, int ldx_dw, int nt, int G, int group,
                                                int KT, float* xgs) {
    const int tpg = group / KT, seg_dw = KT / 4;   // KT/2 columns = KT/4 dwords
    for (int idx = threadIdx.x; idx < nt * G * 2; idx += blockDim.x) {
        const int half = idx & 1, g = (idx >> 1) % G, t = (idx >> 1) / G;
        float s = 0.f;
        for (int tl = 0; tl < tpg; ++tl) {
            const uint32_t* px = xs + t * ldx_dw + ((g * group + tl * KT + half * (KT / 2)) >> 1);
            for (int j = 0; j < seg_dw; ++j) {
                uint32_t v = px[j];
                if constexpr (F16) {
                    __half2 hv = *reinterpret_cast<const __half2*>(&v);
                    s += __low2float(hv) + __high2float(hv);
                } else {
                    s += bf16_lo(v) + bf16_hi(v);
                }
            }
        }
        xgs[idx] = s;   // idx == (t*G + g)*2 + half
    }
}

template <int TT>
__global__ __launch_bounds__(256) void ffn_up_decode_kernel(DecodeArgs a) {
    extern __shared__ uint4 smem[];
    __shared__ float red[2][4][TT][32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    {   // clear this block's slice of y
        const long long total = (long long)a.N * a.H;
        const long long per = (total + gridDim.x - 1) / gridDim.x;
        const long long b0 = (long long)blockIdx.x * per;
        const long long b1 = b0 + per < total ? b0 + per : total;
        for (long long i = b0 + tid; i < b1; i += 256) a.y[i] = 0.f;
    }
    int b = blockIdx.x;
    const int nrout = a.nact * a.rb_r;
    const fate_qexpert* ex;
    int rb, T, sbeg = 0, bits, group, ldh;
    __half* hbuf;
    const bool is_shared = b >= nrout;
    if (!is_shared) {
        const int slot = b / a.rb_r;
        rb = b % a.rb_r;
        const int e = a.order[slot];
        T = a.counts[e];
        if (T == 0) return;
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
    const int I = ex->I;
    if (rb * 32 >= I) return;
    const uint4* w1 = static_cast<const uint4*>(ex->w1);
    const uint4* w3 = static_cast<const uint4*>(ex->w3);
    if (w1 == nullptr || w3 == nullptr) {
        if (tid == 0) atomicOr(a.status, 1);
        return;
    }
    const int H = a.H, nvec = H >> 3, G = H / group;
    const int KT = bits == 4 ? 64 : 32;
    const int tiles_k = H / KT, tpg = group / KT;
    const int n = lane & 31;
    const uint4* wt[2] = {w1 + (size_t)rb * tiles_k * 64 + lane, w3 + (size_t)rb * tiles_k * 64 + lane};
    const __half* sc[2] = {static_cast<const __half*>(ex->s1) + (size_t)(rb * 32 + n) * G,
                           static_cast<const __half*>(ex->s3) + (size_t)(rb * 32 + n) * G};
    const int g_beg = G * wave / 4, g_end = G * (wave + 1) / 4;
    uint32_t* xs = reinterpret_cast<uint32_t*>(smem);
    float* xgs = reinterpret_cast<float*>(smem + (size_t)TT * nvec);
    const uint4* xg = reinterpret_cast<const uint4*>(a.x);

    for (int t0 = 0; t0 < T; t0 += TT) {
        const int nt = min(TT, T - t0);
        __syncthreads();
        for (int idx = tid; idx < nt * nvec; idx += 256) {
            const int t = idx / nvec, c = idx - t * nvec;
            const int tok = is_shared ? t0 + t : a.perm[sbeg + t0 + t] / a.k;
            smem[t * nvec + c] = xg[(size_t)tok * nvec + c];
        }
        __syncthreads();
        group_half_sums<false>(xs, H >> 1, nt, G, group, KT, xgs);
        __syncthreads();
        float out[2][TT];
#pragma unroll
        for (int t = 0; t < TT; ++t) out[0][t] = out[1][t] = 0.f;
        if (bits == 4)
            gemv_rowblock<4, false, TT, 2>(wt, sc, g_beg, g_end, tpg, xs, H >> 1, 0, xgs, G, 0, nt, out);
        else
            gemv_rowblock<8, false, TT, 2>(wt, sc, g_beg, g_end, tpg, xs, H >> 1, 0, xgs, G, 0, nt, out);
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
    }
}

template <int TT>
__global__ __launch_bounds__(256) void ffn_down_decode_kernel(DecodeArgs a) {
    extern __shared__ uint4 smem[];
    __shared__ float red[4][TT][32];
    __shared__ float sgate[TT];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
    const uint4* w2 = static_cast<const uint4*>(ex->w2);
    if (w2 == nullptr) return;   // flagged by the up kernel
    const int KT = bits == 4 ? 64 : 32;
    const int tiles_k = I / KT, tpg = group / KT;
    const int n = lane & 31;
    const uint4* wt[1] = {w2 + (size_t)rb * tiles_k * 64 + lane};
    const __half* sc[1] = {static_cast<const __half*>(ex->s2) + (size_t)(rb * 32 + n) * G};
    const int ng = ge - gb;
    const int g_beg = gb + ng * wave / 4, g_end = gb + ng * (wave + 1) / 4;
    const int Kc = ng * group, kvec = Kc >> 3, k_base = gb * group;
    uint32_t* xs = reinterpret_cast<uint32_t*>(smem);
    float* xgs = reinterpret_cast<float*>(smem + (size_t)TT * kvec);

    for (int t0 = 0; t0 < T; t0 += TT) {
        const int nt = min(TT, T - t0);
        __syncthreads();
        for (int idx = tid; idx < nt * kvec; idx += 256) {
            const int t = idx / kvec, c = idx - t * kvec;
            smem[t * kvec + c] =
                *reinterpret_cast<const uint4*>(hbuf + (size_t)(t0 + t) * ldh + k_base + c * 8);
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
        group_half_sums<true>(xs, Kc >> 1, nt, ng, group, KT, xgs);
        __syncthreads();
        float out[1][TT];
#pragma unroll
        for (int t = 0; t < TT; ++t) out[0][t] = 0.f;
        if (bits == 4)
            gemv_rowblock<4, true, TT, 1>(wt, sc, g_beg, g_end, tpg, xs, Kc >> 1, k_base, xgs, ng, gb, nt, out);
        else
            gemv_rowblock<8, true, TT, 1>(wt, sc, g_beg, g_end, tpg, xs, Kc >> 1, k_base, xgs, ng, gb, nt, out);
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
    // LDS of the up kernel: TT rows of x (bf16) + group sums; of the down kernel: TT rows of an h chunk
    auto lds_up = [&](int tt) {
        size_t g = (size_t)d.H / (size_t)(d.n_shared ? min(d.group, d.shared_group) : d.group);
        return (size_t)tt * d.H * 2 + (size_t)tt * g * 2 * 4;
    };
    const int Gr = d.I_max / d.group, Gs = d.n_shared ? d.I_shared_max / d.shared_group : 0;
    a.nchunk_r = (Gr + 15) / 16; a.cg_r = (Gr + a.nchunk_r - 1) / a.nchunk_r;
    a.nchunk_s = Gs ? (Gs + 15) / 16 : 1; a.cg_s = Gs ? (Gs + a.nchunk_s - 1) / a.nchunk_s : 1;
    auto lds_down = [&](int tt) {
        size_t kr = (size_t)a.cg_r * d.group, ks = d.n_shared ? (size_t)a.cg_s * d.shared_group : 0;
        size_t kc = kr > ks ? kr : ks;
        return (size_t)tt * kc * 2 + (size_t)tt * 16 * 2 * 4 + 256;
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
