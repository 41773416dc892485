// Decode-side expert FFN behind fate_moe_ffn_q: bandwidth-bound dequant-GEMV
// kernels, three launches per layer.
//  up:   a workgroup owns 32 intermediate neurons of one activated expert (or
//        of a shared expert): it streams the matching 32-row blocks of W1 and
//        W3 (device-native 1 KiB tiles, one contiguous KiB per wave load),
//        the four waves splitting the reduction dimension, and writes
//        h = silu(W1 x) * (W3 x) as fp16.
//  down: a workgroup owns 32 output rows of W2 of one expert and a chunk of
//        the reduction dimension, and stores weight * (W2 h) as a partial
//        output row of its own (per pair and chunk; per shared expert, chunk
//        and token).
//  sum:  adds a token's partial rows in a fixed order and writes y - the
//        result does not depend on the order in which workgroups ran.
// Every wave requests its first tiles before anything else and keeps a ring
// of them in flight (decode_device.h), so the HBM stream starts while the
// activations are still being staged in LDS.
#include <hip/hip_fp16.h>
#include "common.h"
#include "qformat.h"
#include "ffn_internal.h"
#include "decode_device.h"

namespace fate {

constexpr int kRing = 8;       // weight tiles in flight per matrix per wave
constexpr int kZpChunkGroups = 64;   // groups of a down chunk the zero-point path keeps activation sums for

__global__ __launch_bounds__(256, 2) void ffn_up_decode_kernel(DecodeArgs a) {
    extern __shared__ uint4 smem[];
    __shared__ float red[2][4][kTokPass][32];
    __shared__ float gsum[kTokPass * kZpMaxGroups];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
        hbuf = a.h_r + (size_t)sbeg * a.ldh_r; ldh = a.ldh_r;
    } else {
        b -= nrout;
        const int s = b / a.rb_s;
        rb = b % a.rb_s;
        ex = a.shared + s;
        T = a.N;
        hbuf = a.h_s + (size_t)s * a.N * a.ldh_s; ldh = a.ldh_s;
    }
    // the width and group of THIS expert's copy (a layer may hold copies of several widths)
    bits = ex->bits; group = ex->group;
    gu4_t w1 = nullptr;
    gu4_t w3 = nullptr;
    if (live) {
        live = rb * 32 < ex->I;
        if (live && !entry_format_ok(bits, group, a.H, ex->I)) {
            if (tid == 0) atomicOr(a.status, 4);
            live = false;
        }
        // zero-points: with the 4- and 2-bit formats, on all three matrices
        if (live && ex->z1 != nullptr &&
            (bits == 8 || ex->z2 == nullptr || ex->z3 == nullptr || a.H / group > kZpMaxGroups)) {
            if (tid == 0) atomicOr(a.status, 4);
            live = false;
        }
        w1 = as_global<uint4>(ex->w1);
        w3 = as_global<uint4>(ex->w3);
        if (live && (w1 == nullptr || w3 == nullptr)) {
            if (tid == 0) atomicOr(a.status, 1);
            live = false;
        }
    }
    if (!live) return;
    const int H = a.H, nvec = H >> 3, G = H / group;
    const int KT = tile_columns(bits);
    const int tiles_k = H / KT, tpg = group / KT;
    const int n = lane & 31, half = lane >> 5;
    const int g_beg = G * wave / 4, g_end = G * (wave + 1) / 4;
    gu4_t wt[2] = {w1 + (size_t)rb * tiles_k * 64 + lane, w3 + (size_t)rb * tiles_k * 64 + lane};
    gu16_t sc[2] = {as_global<uint16_t>(ex->s1) + rb * 32 + n, as_global<uint16_t>(ex->s3) + rb * 32 + n};
    const bool has_z = ex->z1 != nullptr;
    gu16_t zp[2] = {as_global<uint16_t>(has_z ? ex->z1 : ex->s1) + rb * 32 + n,
                    as_global<uint16_t>(has_z ? ex->z3 : ex->s3) + rb * 32 + n};
    const int srows = ex->I;
    const int ldx = H + kLdsPad;                       // halves per LDS row; the last row is all zero
    const int zrow = a.lds_rows - 1;
    _Float16* xs = reinterpret_cast<_Float16*>(smem);
    const uint4* xg = reinterpret_cast<const uint4*>(a.x);

    auto stage_x = [&](int nt, int t0) {
        for (int idx = tid; idx < nt * nvec; idx += 256) {
            const int t = idx / nvec, c = idx - t * nvec;
            const int tok = is_shared ? t0 + t : a.perm[sbeg + t0 + t] / a.k;
            const uint4 v = xg[(size_t)tok * nvec + c];
            *reinterpret_cast<uint4*>(xs + t * ldx + c * 8) = bf16x8_to_f16x8(v);
        }
        if (t0 == 0)
            for (int c = tid; c < (ldx >> 3); c += 256)
                *reinterpret_cast<uint4*>(xs + zrow * ldx + c * 8) = make_uint4(0, 0, 0, 0);
    };
    auto finish = [&](int nt, int t0, float (&out)[2][4]) {
        // lane (half, n) holds tokens 4*half .. 4*half+3 of row n
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            red[0][wave][4 * half + j][n] = out[0][j];
            red[1][wave][4 * half + j][n] = out[1][j];
        }
        __syncthreads();
        if (tid < 32 * nt) {
            const int t = tid >> 5, nn = tid & 31;
            const float a1 = red[0][0][t][nn] + red[0][1][t][nn] + red[0][2][t][nn] + red[0][3][t][nn];
            const float a3 = red[1][0][t][nn] + red[1][1][t][nn] + red[1][2][t][nn] + red[1][3][t][nn];
            const float hv = a1 / (1.0f + expf(-a1)) * a3;
            hbuf[(size_t)(t0 + t) * ldh + rb * 32 + nn] = __float2half(hv);
        }
    };

#define FATE_UP_BODY_(BITS, TPG, ZP)                                                                     \
    {                                                                                                     \
        TileRing<2, kRing, TPG, ZP> ring;                                                                 \
        ring_start<2, kRing, TPG, ZP>(ring, wt, sc, srows, g_beg, g_end, zp);                             \
        for (int t0 = 0; t0 < T; t0 += kTokPass) {                                                        \
            const int nt = min(kTokPass, T - t0);                                                         \
            if (t0 > 0) {                                                                                 \
                __syncthreads();                                                                          \
                ring_start<2, kRing, TPG, ZP>(ring, wt, sc, srows, g_beg, g_end, zp);                     \
            }                                                                                             \
            stage_x(nt, t0);                                                                              \
            __syncthreads();                                                                              \
            if (ZP) {                                                                                     \
                stage_group_sums(xs, ldx, nt, G, group, gsum);                                            \
                __syncthreads();                                                                          \
            }                                                                                             \
            float out[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};                               \
            const int arow = n < nt ? n : zrow;                                                           \
            ring_run<BITS, TPG, 2, kRing, ZP>(ring, wt, sc, srows, g_beg, g_end,                          \
                                              xs + arow * ldx + half * (QFmt<BITS>::KT / 2), 0, out, zp,  \
                                              gsum + 4 * half * G, G, 0);                                 \
            finish(nt, t0, out);                                                                          \
        }                                                                                                 \
    }
#define FATE_UP_BODY(BITS, TPG) FATE_UP_BODY_(BITS, TPG, false)
#define FATE_UP_BODY_Z(BITS, TPG) FATE_UP_BODY_(BITS, TPG, true)
    if (has_z) {
        FATE_FORMAT_SWITCH_ZP(bits, tpg, FATE_UP_BODY_Z)
    } else {
        FATE_FORMAT_SWITCH_ALL(bits, tpg, FATE_UP_BODY)
    }
#undef FATE_UP_BODY
#undef FATE_UP_BODY_Z
#undef FATE_UP_BODY_
}

__global__ __launch_bounds__(256) void ffn_down_decode_kernel(DecodeArgs a) {
    extern __shared__ uint4 smem[];
    __shared__ float red[4][kTokPass][32];
    __shared__ float sgate[kTokPass];
    __shared__ float gsum[kTokPass * kZpChunkGroups];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nrb = a.H >> 5;
    int b = blockIdx.x;
    const int nrout = a.nact * nrb * a.nchunk_r;
    const fate_qexpert* ex;
    int rb, ch, cg, T, sbeg = 0, bits, group, ldh, sidx = 0;
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
        hbuf = a.h_r + (size_t)sbeg * a.ldh_r; ldh = a.ldh_r;
    } else {
        b -= nrout;
        const int s = b / (nrb * a.nchunk_s);
        const int rem = b - s * (nrb * a.nchunk_s);
        rb = rem / a.nchunk_s; ch = rem - rb * a.nchunk_s; cg = a.cg_s;
        ex = a.shared + s;
        sidx = s;
        T = a.N;
        hbuf = a.h_s + (size_t)s * a.N * a.ldh_s; ldh = a.ldh_s;
    }
    bits = ex->bits; group = ex->group;
    // this block's partial output rows: per pair (sorted order) and chunk, or per shared expert, chunk and token
    const int nchunk = is_shared ? a.nchunk_s : a.nchunk_r;
    auto part_row = [&](int t) -> float* {
        return is_shared ? a.part_s + (((size_t)sidx * nchunk + ch) * a.N + t) * a.H
                         : a.part_r + ((size_t)(sbeg + t) * nchunk + ch) * a.H;
    };
    auto nothing = [&]() {      // a block without weights to multiply still owes its rows: zeros
        for (int i = tid; i < T * 32; i += 256) part_row(i >> 5)[rb * 32 + (i & 31)] = 0.f;
    };
    if (!entry_format_ok(bits, group, a.H, ex->I)) {          // flagged by the up kernel
        nothing();
        return;
    }
    // the launch cut the reduction dimension into chunks of cg groups of the descriptor's group size
    cg = cg * (is_shared ? a.group_s : a.group_r) / group;
    const int I = ex->I, G = I / group;
    const int gb = ch * cg, ge = min(G, gb + cg);
    gu4_t w2 = as_global<uint4>(ex->w2);
    const bool has_z = ex->z1 != nullptr;
    const bool bad_z = has_z && (bits == 8 || ex->z2 == nullptr || ex->z3 == nullptr || a.H / group > kZpMaxGroups ||
                                 ge - gb > kZpChunkGroups);
    if (bad_z && tid == 0) atomicOr(a.status, 4);
    if (gb >= ge || w2 == nullptr || ex->w1 == nullptr || ex->w3 == nullptr || bad_z) {   // (a missing expert is flagged by the up kernel)
        nothing();
        return;
    }
    const int KT = tile_columns(bits);
    const int tiles_k = I / KT, tpg = group / KT;
    const int n = lane & 31, half = lane >> 5;
    gu4_t wt[1] = {w2 + (size_t)rb * tiles_k * 64 + lane};
    gu16_t sc[1] = {as_global<uint16_t>(ex->s2) + rb * 32 + n};
    gu16_t zp[1] = {as_global<uint16_t>(has_z ? ex->z2 : ex->s2) + rb * 32 + n};
    const int srows = a.H;
    const int ng = ge - gb;
    const int g_beg = gb + ng * wave / 4, g_end = gb + ng * (wave + 1) / 4;
    const int Kc = ng * group, kvec = Kc >> 3, k_base = gb * group;
    const int ldx = Kc + kLdsPad;
    const int zrow = a.lds_rows - 1;
    _Float16* xs = reinterpret_cast<_Float16*>(smem);

    auto stage_h = [&](int nt, int t0) {
        for (int idx = tid; idx < nt * kvec; idx += 256) {
            const int t = idx / kvec, c = idx - t * kvec;
            *reinterpret_cast<uint4*>(xs + t * ldx + c * 8) =
                *reinterpret_cast<const uint4*>(hbuf + (size_t)(t0 + t) * ldh + k_base + c * 8);
        }
        if (t0 == 0)
            for (int c = tid; c < (ldx >> 3); c += 256)
                *reinterpret_cast<uint4*>(xs + zrow * ldx + c * 8) = make_uint4(0, 0, 0, 0);
        if (is_shared && a.shared_gate != nullptr) {
            const int nvec = a.H >> 3;
            for (int t = wave; t < nt; t += 4) {
                const float g = wave_sigmoid_dot_bf16(reinterpret_cast<const uint4*>(a.x) + (size_t)(t0 + t) * nvec,
                                                      reinterpret_cast<const uint4*>(a.shared_gate), nvec);
                if (lane == 0) sgate[t] = g;
            }
        }
    };
    auto finish = [&](int nt, int t0, float (&out)[1][4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) red[wave][4 * half + j][n] = out[0][j];
        __syncthreads();
        if (tid < 32 * nt) {
            const int t = tid >> 5, nn = tid & 31;
            const float v = red[0][t][nn] + red[1][t][nn] + red[2][t][nn] + red[3][t][nn];
            float wgt;
            if (is_shared) wgt = a.shared_gate ? sgate[t] : 1.0f;
            else wgt = a.topk_w[a.perm[sbeg + t0 + t]];
            part_row(t0 + t)[rb * 32 + nn] = wgt * v;
        }
    };

#define FATE_DOWN_BODY_(BITS, TPG, ZP)                                                                   \
    {                                                                                                     \
        TileRing<1, kRing, TPG, ZP> ring;                                                                 \
        ring_start<1, kRing, TPG, ZP>(ring, wt, sc, srows, g_beg, g_end, zp);                             \
        for (int t0 = 0; t0 < T; t0 += kTokPass) {                                                        \
            const int nt = min(kTokPass, T - t0);                                                         \
            if (t0 > 0) {                                                                                 \
                __syncthreads();                                                                          \
                ring_start<1, kRing, TPG, ZP>(ring, wt, sc, srows, g_beg, g_end, zp);                     \
            }                                                                                             \
            stage_h(nt, t0);                                                                              \
            __syncthreads();                                                                              \
            if (ZP) {                                                                                     \
                stage_group_sums(xs, ldx, nt, ng, group, gsum);                                           \
                __syncthreads();                                                                          \
            }                                                                                             \
            float out[1][4] = {{0.f, 0.f, 0.f, 0.f}};                                                     \
            const int arow = n < nt ? n : zrow;                                                           \
            ring_run<BITS, TPG, 1, kRing, ZP>(ring, wt, sc, srows, g_beg, g_end,                          \
                                              xs + arow * ldx + half * (QFmt<BITS>::KT / 2), k_base, out, \
                                              zp, gsum + 4 * half * ng, ng, gb);                          \
            finish(nt, t0, out);                                                                          \
        }                                                                                                 \
    }
#define FATE_DOWN_BODY(BITS, TPG) FATE_DOWN_BODY_(BITS, TPG, false)
#define FATE_DOWN_BODY_Z(BITS, TPG) FATE_DOWN_BODY_(BITS, TPG, true)
    if (has_z) {
        FATE_FORMAT_SWITCH_ZP(bits, tpg, FATE_DOWN_BODY_Z)
    } else {
        FATE_FORMAT_SWITCH_ALL(bits, tpg, FATE_DOWN_BODY)
    }
#undef FATE_DOWN_BODY
#undef FATE_DOWN_BODY_Z
#undef FATE_DOWN_BODY_
}

// y[t,:] = sum over the token's pairs (in pair order) and their chunks, then over the shared experts and theirs
__global__ __launch_bounds__(256) void ffn_sum_decode_kernel(DecodeArgs a, void* y_out, int y_is_fp32) {
    const int t = blockIdx.x;
    const int H = a.H;
    for (int c = threadIdx.x; c < (H >> 2); c += 256) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        auto add = [&](const float* row) {
            const float4 v = reinterpret_cast<const float4*>(row)[c];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        };
        for (int j = 0; j < a.k; ++j) {
            const int pos = a.inv_perm[t * a.k + j];
            if (pos < 0) continue;                       // a pair whose expert id was out of range
            for (int ch = 0; ch < a.nchunk_r; ++ch) add(a.part_r + ((size_t)pos * a.nchunk_r + ch) * H);
        }
        for (int s = 0; s < a.n_shared; ++s)
            for (int ch = 0; ch < a.nchunk_s; ++ch) add(a.part_s + (((size_t)s * a.nchunk_s + ch) * a.N + t) * H);
        if (y_is_fp32) {
            reinterpret_cast<float4*>(static_cast<float*>(y_out) + (size_t)t * H)[c] = acc;
        } else {
            const uint32_t lo = f32_to_bf16_bits(acc.x) | (f32_to_bf16_bits(acc.y) << 16);
            const uint32_t hi = f32_to_bf16_bits(acc.z) | (f32_to_bf16_bits(acc.w) << 16);
            reinterpret_cast<uint2*>(static_cast<uint16_t*>(y_out) + (size_t)t * H)[c] = make_uint2(lo, hi);
        }
    }
}

constexpr size_t kLdsMax = 96 * 1024;

fate_status launch_ffn_decode(hipStream_t st, const fate_ffn_desc& d, DecodeArgs a, void* y_out) {
    if (!decode_group_ok(d.bits, d.group) || (d.n_shared && !decode_group_ok(d.shared_bits, d.shared_group)))
        FATE_FAIL(FATE_ESHAPE, "decode path: group must be 64, 128 or 256 (int4) / 64 or 128 (int8)");
    const int Gr = d.I_max / d.group, Gs = d.n_shared ? d.I_shared_max / d.shared_group : 0;
    a.nchunk_r = decode_down_chunks(Gr); a.cg_r = (Gr + a.nchunk_r - 1) / a.nchunk_r;
    a.nchunk_s = decode_down_chunks(Gs); a.cg_s = Gs ? (Gs + a.nchunk_s - 1) / a.nchunk_s : 1;
    // LDS: the activation rows of one pass + one zero row, fp16, padded
    a.lds_rows = (d.N < kTokPass ? d.N : kTokPass) + 1;
    const size_t lu = (size_t)a.lds_rows * (d.H + kLdsPad) * 2;
    const size_t kr = (size_t)a.cg_r * d.group, ks = d.n_shared ? (size_t)a.cg_s * d.shared_group : 0;
    const size_t ld = (size_t)a.lds_rows * ((kr > ks ? kr : ks) + kLdsPad) * 2;
    if (lu > kLdsMax || ld > kLdsMax) FATE_FAIL(FATE_ESHAPE, "H = %d too large for the decode kernels", d.H);
    static bool attr_done = false;
    if (!attr_done) {
        FATE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_up_decode_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax));
        FATE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_down_decode_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax));
        attr_done = true;
    }
    a.nact = min(d.E, d.N * d.k);
    a.rb_r = d.I_max / 32;
    a.rb_s = d.n_shared ? d.I_shared_max / 32 : 0;
    const int grid_up = a.nact * a.rb_r + d.n_shared * a.rb_s;
    const int nrb = d.H / 32;
    const int grid_down = a.nact * nrb * a.nchunk_r + d.n_shared * nrb * a.nchunk_s;
    ffn_up_decode_kernel<<<grid_up, 256, lu, st>>>(a);
    ffn_down_decode_kernel<<<grid_down, 256, ld, st>>>(a);
    FATE_HIP(hipGetLastError());
    ffn_sum_decode_kernel<<<d.N, 256, 0, st>>>(a, y_out, d.y_is_fp32);
    FATE_HIP(hipGetLastError());
    return FATE_OK;
}

}  // namespace fate
