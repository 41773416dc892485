// Gate routing, cross-layer prediction, permutation: kernels and C entry points.
//
// fate_gate_route / fate_cross_layer_predict: one wavefront per token row.
// The wave keeps its token rows in LDS, streams the gate matrix (L2
// resident) row by row, reduces each logit with wavefront shuffles, then
// does the softmax and the top-m selection in registers.
//
// fate_route_fused: decode-side variant.  With a handful of tokens the gate
// matrices (2 x E rows) are the only sizeable data, so one wave takes one gate
// row for all tokens and the rows are spread over the chip; the workgroup
// that finishes last (ticket counter) does softmax, selection, popularity
// and the permutation for all tokens.
#include "common.h"
#include "route_device.h"

namespace fate {

__global__ void fill_i32_kernel(int32_t* p, int n, int32_t v) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// 4 waves per block, TPW token rows per wave.
template <int TPW>
__global__ __launch_bounds__(256) void route_rows_kernel(const uint16_t* __restrict__ x,
                                                         const uint16_t* __restrict__ Wg,
                                                         const float* __restrict__ bias, int N, int H, int E,
                                                         int m, int renorm, int32_t* __restrict__ ids,
                                                         float* __restrict__ w, float* __restrict__ probs,
                                                         int32_t* __restrict__ pop) {
    extern __shared__ uint4 smem[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nvec = H >> 3;
    const int tok0 = (blockIdx.x * 4 + wave) * TPW;
    uint4* xw = smem + (size_t)wave * TPW * nvec;
    float* zw = reinterpret_cast<float*>(smem + (size_t)4 * TPW * nvec) + (size_t)wave * TPW * E;

    for (int t = 0; t < TPW; ++t) {
        int tok = tok0 + t;
        const uint4* xr = reinterpret_cast<const uint4*>(x) + (size_t)tok * nvec;
        for (int c = lane; c < nvec; c += 64) xw[t * nvec + c] = (tok < N) ? xr[c] : make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
    for (int e = 0; e < E; ++e) {
        float acc[TPW];
#pragma unroll
        for (int t = 0; t < TPW; ++t) acc[t] = 0.f;
        const uint4* wr = reinterpret_cast<const uint4*>(Wg) + (size_t)e * nvec;
        for (int c = lane; c < nvec; c += 64) {
            uint4 wv = wr[c];
#pragma unroll
            for (int t = 0; t < TPW; ++t) acc[t] = dot8_bf16(xw[t * nvec + c], wv, acc[t]);
        }
        float b = bias ? bias[e] : 0.f;
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            float s = wave_sum(acc[t]);
            if (lane == 0) zw[t * E + e] = s + b;
        }
    }
    __syncthreads();
    for (int t = 0; t < TPW; ++t) {
        int tok = tok0 + t;
        if (tok < N)
            wave_softmax_topm(zw + t * E, E, m, renorm, ids + (size_t)tok * m, w + (size_t)tok * m,
                              probs ? probs + (size_t)tok * E : nullptr, pop);
    }
}

// Many tokens (prefill): the gate is a small GEMM, z[N,E] = x[N,H] . Wg[E,H]^T, done on the matrix
// cores.  A workgroup (8 waves) owns 32 tokens; wave w takes expert tile (w & 1) of a pair of
// 32-expert tiles and quarter (w >> 1) of the reduction dimension; the quarters add up in LDS.  Both operands are row-major with the
// reduction dimension contiguous, which is the register layout of v_mfma_f32_32x32x16_bf16 as it
// stands: lane (half, r) holds 8 consecutive elements of row r - 16 bytes straight from memory.
// bf16 products are exact in fp32; accumulation is fp32.  The logits meet in LDS, then one wave
// per token does softmax and selection as in the other kernels.
struct RouteSecond {             // arguments of the second gate (grid.y = 2); unused when grid.y = 1
    const uint16_t* Wg; const float* bias; int m; int32_t* ids; float* w; int32_t* pop;
    int32_t* pop_part;           // [workgroups][E]: when set, a workgroup leaves its counts here (plain stores)
                                 // for the permutation kernel to add up, and pop needs neither zeroing nor atomics
};
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float rf32x16_t;
constexpr int kGemmTok = 32;

__global__ __launch_bounds__(512) void route_mfma_kernel(const uint16_t* __restrict__ x,
                                                         const uint16_t* __restrict__ Wg,
                                                         const float* __restrict__ bias, int N, int H, int E,
                                                         int m, int renorm, int32_t* __restrict__ ids,
                                                         float* __restrict__ w, float* __restrict__ probs,
                                                         int32_t* __restrict__ pop, int ntok, RouteSecond g2) {
    // ntok <= 32 tokens per workgroup: with few tokens in the call, fewer rows of the 32-row
    // product are live but more workgroups share the work (each still reads all of Wg)
    extern __shared__ float zs[];                 // [4 quarters][32 tokens][Epad]
    // popularity counts of this workgroup's tokens: added up here first, so that the device-wide
    // histogram takes one atomic per workgroup and expert instead of one per token and expert
    // (atomics on one address are served one after the other, and popular experts are popular)
    __shared__ int32_t pop_s[kMaxE];
    int32_t* pop_part = nullptr;
    if (blockIdx.y == 1) {                        // the second gate of the same launch (next layer's)
        Wg = g2.Wg; bias = g2.bias; m = g2.m; renorm = 0; ids = g2.ids; w = g2.w; probs = nullptr; pop = g2.pop;
        pop_part = g2.pop_part;
    }
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, half = lane >> 5;
    const int etile = wave & 1, kq = wave >> 1;
    const int Epad = (E + 63) & ~63;
    const int t0 = blockIdx.x * ntok;
    const int tok = n < ntok ? t0 + n : N;        // rows past ntok: no token
    const int kbeg = kq * (H >> 2), kend = kbeg + (H >> 2);

    // Rows without a token and columns without an expert read row 0 instead (their products are
    // never looked at): every load is unconditional, so the compiler's waits count the loads
    // still in flight and the next chunk's operands travel under this chunk's products.
    const uint4* xr = reinterpret_cast<const uint4*>(x + (size_t)(tok < N ? tok : 0) * H) + half;
    for (int e0 = 0; e0 < E; e0 += 64) {
        const int e = e0 + etile * 32 + n;
        const uint4* wr = reinterpret_cast<const uint4*>(Wg + (size_t)(e < E ? e : 0) * H) + half;
        rf32x16_t acc;
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j] = 0.f;
        // chunks of eight matrix-core steps (H % 1024 == 0: a quarter of K is a whole number of
        // pairs of chunks)
        constexpr int kStep = 8;
        uint4 av[2][kStep], bv[2][kStep];
        auto request = [&](uint4 (&a)[kStep], uint4 (&b)[kStep], int k) {
#pragma unroll
            for (int u = 0; u < kStep; ++u) {
                a[u] = xr[(k + 16 * u) >> 3];
                b[u] = wr[(k + 16 * u) >> 3];
            }
        };
        auto multiply = [&](const uint4 (&a)[kStep], const uint4 (&b)[kStep]) {
#pragma unroll
            for (int u = 0; u < kStep; ++u)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a[u]),
                                                              __builtin_bit_cast(bf16x8_t, b[u]), acc, 0, 0, 0);
        };
        request(av[0], bv[0], kbeg);
        for (int k = kbeg; k < kend; k += 2 * 16 * kStep) {
            request(av[1], bv[1], k + 16 * kStep);
            multiply(av[0], bv[0]);
            // the last request of the row runs past this wave's quarter by one chunk: clamped to stay inside the row
            request(av[0], bv[0], k + 2 * 16 * kStep < kend ? k + 2 * 16 * kStep : kbeg);
            multiply(av[1], bv[1]);
        }
        // lane (half, n) holds expert column n, token rows 8*(j/4) + 4*half + j%4
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int t = 8 * (j >> 2) + 4 * half + (j & 3);
            zs[((size_t)kq * kGemmTok + t) * Epad + e0 + etile * 32 + n] = acc[j];
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < ntok * E; i += 512) {
        const int t = i / E, e = i - t * E;
        const size_t o = (size_t)t * Epad + e, q = (size_t)kGemmTok * Epad;
        zs[o] = ((zs[o] + zs[o + q]) + (zs[o + 2 * q] + zs[o + 3 * q])) + (bias ? bias[e] : 0.f);
    }
    if (pop)
        for (int i = threadIdx.x; i < E; i += 512) pop_s[i] = 0;
    __syncthreads();
    for (int t = wave; t < ntok; t += 8) {
        const int tk = t0 + t;
        if (tk < N)
            wave_softmax_topm(zs + (size_t)t * Epad, E, m, renorm, ids + (size_t)tk * m, w + (size_t)tk * m,
                              probs ? probs + (size_t)tk * E : nullptr, pop ? pop_s : nullptr);
    }
    if (pop) {
        __syncthreads();
        if (pop_part) {
            for (int i = threadIdx.x; i < E; i += 512) pop_part[(size_t)blockIdx.x * E + i] = pop_s[i];
        } else {
            for (int i = threadIdx.x; i < E; i += 512)
                if (pop_s[i]) atomicAdd(&pop[i], pop_s[i]);
        }
    }
}

__global__ __launch_bounds__(1024) void permute_kernel(const int32_t* __restrict__ ids, int P, int E,
                                                       int32_t* counts, int32_t* offsets, int32_t* perm,
                                                       int32_t* inv_perm, int32_t* order,
                                                       const int32_t* __restrict__ pop_part, int nparts,
                                                       int32_t* __restrict__ pop_out) {
    __shared__ int32_t sm[kPermSmemInts];
    if (pop_part) {
        // predicted popularity: the routing workgroups' partial histograms [nparts][E] added up
        // (lane = expert within a group of 64, wave = every 16th partial row)
        __shared__ int32_t hist[kMaxE];
        const int lane = threadIdx.x & 63, row = threadIdx.x >> 6;
        for (int i = threadIdx.x; i < E; i += 1024) hist[i] = 0;
        __syncthreads();
        for (int e = lane; e < E; e += 64) {
            int sum = 0;
            for (int p = row; p < nparts; p += 16) sum += pop_part[(size_t)p * E + e];
            if (sum) atomicAdd(&hist[e], sum);
        }
        __syncthreads();
        for (int i = threadIdx.x; i < E; i += 1024) pop_out[i] = hist[i];
    }
    if (P <= 64) {
        if (threadIdx.x < 64) wave_permute_small(ids, P, E, counts, offsets, perm, inv_perm, order);
        return;
    }
    block_permute(ids, P, E, counts, offsets, perm, inv_perm, order, sm);
}

// ---- fused decode-side routing --------------------------------------------
// workspace: [0] ticket counter (int32, zero between calls), then at byte 256
// the logits zbuf[2][N][E] fp32.
__global__ __launch_bounds__(256) void route_fused_kernel(FusedRouteArgs a, int32_t* ticket) {
    __shared__ FusedRouteSmem sm;
    __shared__ int32_t sm_perm[kPermSmemInts];
    __shared__ int sm_last;
    fused_gate_rows(a, blockIdx.x, ZbufStore{a.zbuf, a.N, a.E});
    wait_own_stores();      // this wave's device-scope logit stores have been acknowledged
    __syncthreads();        // ... and so have every other wave's
    if (threadIdx.x == 0) sm_last = (atomicAdd(ticket, 1) == (int)gridDim.x - 1);
    __syncthreads();
    if (!sm_last) return;
    fused_select(a, sm, sm_perm, ZbufLoad{a.zbuf, a.N, a.E});
    if (threadIdx.x == 0) *ticket = 0;
}

static fate_status check_route_args(const void* x, const void* Wg, const float* bias, int N, int H, int E, int k,
                                    int m, const void* ids, const void* w) {
    if (N < 0) FATE_FAIL(FATE_EINVAL, "N = %d < 0", N);
    if (E < 1 || E > kMaxE) FATE_FAIL(FATE_ESHAPE, "E = %d outside [1, %d]", E, kMaxE);
    if (H < 64 || (H % 64) != 0) FATE_FAIL(FATE_ESHAPE, "H = %d must be a positive multiple of 64", H);
    if (k < 1 || k > m) FATE_FAIL(FATE_EINVAL, "need 1 <= k <= m (k = %d, m = %d)", k, m);
    if (m > E || m > kMaxM) FATE_FAIL(FATE_EINVAL, "m = %d exceeds min(E, %d)", m, kMaxM);
    if (N == 0) return FATE_OK;
    FATE_CHECK_PTR(x);
    FATE_CHECK_PTR(Wg);
    FATE_CHECK_PTR_OPT(bias);
    FATE_CHECK_PTR(ids);
    FATE_CHECK_PTR(w);
    return FATE_OK;
}

static int pick_tpw(int N, int H, int E) {
    if (N < 256) return 1;
    for (int tpw = 4; tpw > 1; tpw >>= 1)
        if ((size_t)4 * tpw * (2 * (size_t)H + 4 * (size_t)E) <= 65536) return tpw;
    return 1;
}

// tokens per workgroup of the gate GEMM: enough workgroups for the device before the tile is
// filled with tokens
static int route_mfma_ntok(int N) { return N > 4096 ? 32 : (N > 1024 ? 16 : 8); }

static fate_status launch_route_mfma(hipStream_t st, const void* x, const void* Wg, const float* bias, int N, int H,
                                     int E, int m, bool renorm, int32_t* ids, float* w, float* probs, int32_t* pop,
                                     RouteSecond second, int ngates) {
    const size_t lds_g = (size_t)4 * kGemmTok * ((E + 63) & ~63) * sizeof(float);
    static bool attr_done = false;
    if (!attr_done) {
        FATE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(route_mfma_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 4 * kGemmTok * kMaxE * 4));
        attr_done = true;
    }
    const int ntok = route_mfma_ntok(N);
    route_mfma_kernel<<<dim3((N + ntok - 1) / ntok, ngates), 512, lds_g, st>>>(
        static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(Wg), bias, N, H, E, m, renorm, ids, w, probs, pop,
        ntok, second);
    FATE_HIP(hipGetLastError());
    return FATE_OK;
}

static fate_status launch_route_rows(hipStream_t st, const void* x, const void* Wg, const float* bias, int N,
                                     int H, int E, int m, int renorm, int32_t* ids, float* w, float* probs,
                                     int32_t* pop) {
    auto xs = static_cast<const uint16_t*>(x);
    auto ws = static_cast<const uint16_t*>(Wg);
    if (N >= 64 && H % 1024 == 0)     // prefill-sized batches: gate GEMM on the matrix cores
        return launch_route_mfma(st, x, Wg, bias, N, H, E, m, renorm, ids, w, probs, pop, RouteSecond{}, 1);
    const int tpw = pick_tpw(N, H, E);
    const size_t lds = (size_t)4 * tpw * (2 * (size_t)H + 4 * (size_t)E);
    if (lds > 65536) FATE_FAIL(FATE_ESHAPE, "H = %d, E = %d need %zu bytes of LDS (> 64 KiB)", H, E, lds);
    const int grid = (N + 4 * tpw - 1) / (4 * tpw);
    switch (tpw) {
        case 4: route_rows_kernel<4><<<grid, 256, lds, st>>>(xs, ws, bias, N, H, E, m, renorm, ids, w, probs, pop); break;
        case 2: route_rows_kernel<2><<<grid, 256, lds, st>>>(xs, ws, bias, N, H, E, m, renorm, ids, w, probs, pop); break;
        default: route_rows_kernel<1><<<grid, 256, lds, st>>>(xs, ws, bias, N, H, E, m, renorm, ids, w, probs, pop); break;
    }
    FATE_HIP(hipGetLastError());
    return FATE_OK;
}

}  // namespace fate

using namespace fate;

extern "C" fate_status fate_gate_route(void* stream, const void* x_bf16, const void* Wg_bf16, const float* bias,
                                       int N, int H, int E, int k, int renorm, int32_t* topk_ids, float* topk_w,
                                       float* probs) {
    fate_status s = check_route_args(x_bf16, Wg_bf16, bias, N, H, E, k, k, topk_ids, topk_w);
    if (s != FATE_OK) return s;
    FATE_CHECK_PTR_OPT(probs);
    if (N == 0) return FATE_OK;
    return launch_route_rows(static_cast<hipStream_t>(stream), x_bf16, Wg_bf16, bias, N, H, E, k, renorm != 0,
                             topk_ids, topk_w, probs, nullptr);
}

extern "C" fate_status fate_cross_layer_predict(void* stream, const void* x_bf16, const void* Wg_next_bf16,
                                                const float* bias_next, int N, int H, int E, int k, int m,
                                                int32_t* pred_ids, float* pred_w, int32_t* pred_pop) {
    fate_status s = check_route_args(x_bf16, Wg_next_bf16, bias_next, N, H, E, k, m, pred_ids, pred_w);
    if (s != FATE_OK) return s;
    if (pred_pop == nullptr) FATE_FAIL(FATE_EINVAL, "pred_pop is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    fill_i32_kernel<<<(E + 255) / 256, 256, 0, st>>>(pred_pop, E, 0);
    FATE_HIP(hipGetLastError());
    if (N == 0) return FATE_OK;
    return launch_route_rows(st, x_bf16, Wg_next_bf16, bias_next, N, H, E, m, 0, pred_ids, pred_w, nullptr,
                             pred_pop);
}

extern "C" fate_status fate_permute(void* stream, const int32_t* topk_ids, int N, int k, int E, int32_t* counts,
                                    int32_t* offsets, int32_t* perm, int32_t* inv_perm, int32_t* expert_order) {
    if (N < 0 || k < 1) FATE_FAIL(FATE_EINVAL, "need N >= 0 and k >= 1 (N = %d, k = %d)", N, k);
    if (E < 1 || E > kMaxE) FATE_FAIL(FATE_ESHAPE, "E = %d outside [1, %d]", E, kMaxE);
    if ((long long)N * k > 0x7fffffffLL) FATE_FAIL(FATE_ESHAPE, "N*k overflows int32");
    if (counts == nullptr || offsets == nullptr || expert_order == nullptr)
        FATE_FAIL(FATE_EINVAL, "counts, offsets and expert_order must not be NULL");
    if (N > 0 && (topk_ids == nullptr || perm == nullptr || inv_perm == nullptr))
        FATE_FAIL(FATE_EINVAL, "topk_ids, perm and inv_perm must not be NULL when N > 0");
    permute_kernel<<<1, 1024, 0, static_cast<hipStream_t>(stream)>>>(topk_ids, N * k, E, counts, offsets, perm,
                                                                    inv_perm, expert_order, nullptr, 0, nullptr);
    FATE_HIP(hipGetLastError());
    return FATE_OK;
}

extern "C" fate_status fate_route_fused_workspace(int N, int E, size_t* bytes) {
    if (bytes == nullptr) FATE_FAIL(FATE_EINVAL, "bytes is NULL");
    if (N < 0 || E < 1 || E > kMaxE) FATE_FAIL(FATE_EINVAL, "bad N or E");
    *bytes = 256 + (size_t)2 * (size_t)(N > 0 ? N : 1) * E * sizeof(float);
    return FATE_OK;
}

extern "C" fate_status fate_route_fused(void* stream, const void* x_bf16, const void* Wg_bf16, const float* bias,
                                        const void* Wg_next_bf16, const float* bias_next, int N, int H, int E,
                                        int k, int m, int renorm, int32_t* topk_ids, float* topk_w,
                                        int32_t* pred_ids, float* pred_w, int32_t* pred_pop, int32_t* counts,
                                        int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                                        int32_t* expert_order, void* workspace, size_t workspace_bytes) {
    fate_status s = check_route_args(x_bf16, Wg_bf16, bias, N, H, E, k, m, topk_ids, topk_w);
    if (s != FATE_OK) return s;
    const bool big = N >= 64 && H % 1024 == 0;     // both gate products in one launch on the matrix cores
    if (N < 1 || (N > kFusedMaxN && !big))
        FATE_FAIL(FATE_ESHAPE, "fused routing needs 1 <= N <= %d, or N >= 64 with H a multiple of 1024 (N = %d, H = %d)",
                  kFusedMaxN, N, H);
    if (Wg_next_bf16) {
        FATE_CHECK_PTR(Wg_next_bf16);
        FATE_CHECK_PTR_OPT(bias_next);
        if (!pred_ids || !pred_w || !pred_pop) FATE_FAIL(FATE_EINVAL, "pred outputs must not be NULL");
    }
    if (!counts || !offsets || !perm || !inv_perm || !expert_order)
        FATE_FAIL(FATE_EINVAL, "permutation outputs must not be NULL");
    size_t need = 0;
    fate_route_fused_workspace(N, E, &need);
    if (workspace == nullptr || workspace_bytes < need)
        FATE_FAIL(FATE_EWORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    FATE_CHECK_PTR(workspace);
    if (big) {
        hipStream_t st = static_cast<hipStream_t>(stream);
        // the workgroups' popularity counts go through the workspace and are added up by the
        // permutation kernel: no zeroing launch, no atomics on the device-wide histogram
        const int ntok = route_mfma_ntok(N), nparts = (N + ntok - 1) / ntok;
        int32_t* pop_part = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + 256);
        s = launch_route_mfma(st, x_bf16, Wg_bf16, bias, N, H, E, k, renorm != 0, topk_ids, topk_w, nullptr, nullptr,
                              RouteSecond{static_cast<const uint16_t*>(Wg_next_bf16), bias_next, m, pred_ids, pred_w,
                                          pred_pop, pop_part},
                              Wg_next_bf16 ? 2 : 1);
        if (s != FATE_OK) return s;
        permute_kernel<<<1, 1024, 0, st>>>(topk_ids, N * k, E, counts, offsets, perm, inv_perm, expert_order,
                                           Wg_next_bf16 ? pop_part : nullptr, nparts, pred_pop);
        FATE_HIP(hipGetLastError());
        return FATE_OK;
    }
    const int nrows = Wg_next_bf16 ? 2 * E : E;
    const int grid = (nrows + 3) / 4;
    FusedRouteArgs a{static_cast<const uint16_t*>(x_bf16), static_cast<const uint16_t*>(Wg_bf16), bias,
                     static_cast<const uint16_t*>(Wg_next_bf16), bias_next, N, H, E, k, m, renorm != 0,
                     topk_ids, topk_w, pred_ids, pred_w, pred_pop, counts, offsets, perm, inv_perm, expert_order,
                     reinterpret_cast<float*>(static_cast<char*>(workspace) + 256)};
    route_fused_kernel<<<grid, 256, 0, static_cast<hipStream_t>(stream)>>>(a, static_cast<int32_t*>(workspace));
    FATE_HIP(hipGetLastError());
    return FATE_OK;
}
