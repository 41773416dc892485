// fate_moe_layer_decode: the one-item-per-block kernels of every pair of weight formats, the
// host side (checks, launch geometry, dispatch) and the small reduction kernel that adds up the
// partial output rows.  The looping kernels live in layer_decode_loop_r*.hip.
#include "layer_decode_impl.h"
#include "layer_decode_b1.h"

namespace fate {

fate_status launch_layer_loop_4_1(hipStream_t, int, int, int, int, int, const LayerArgs&);
fate_status launch_layer_loop_4_2(hipStream_t, int, int, int, int, int, const LayerArgs&);
fate_status launch_layer_loop_4_4(hipStream_t, int, int, int, int, int, const LayerArgs&);
fate_status launch_layer_loop_8_2(hipStream_t, int, int, int, int, int, const LayerArgs&);
fate_status launch_layer_loop_8_4(hipStream_t, int, int, int, int, int, const LayerArgs&);
int layer_loop_blocks_per_cu_4_1(int, int, int, int);
int layer_loop_blocks_per_cu_4_2(int, int, int, int);
int layer_loop_blocks_per_cu_4_4(int, int, int, int);
int layer_loop_blocks_per_cu_8_2(int, int, int, int);
int layer_loop_blocks_per_cu_8_4(int, int, int, int);

// y[t] = sum over the k pairs of token t and the 32-neuron blocks of their experts, plus the
// shared experts' blocks.  A workgroup owns 32 consecutive outputs of one token; one wave load
// covers two partial rows (a half-wave each), the 16 waves take rows in turn with all their
// loads in flight at once, and the partial sums meet in LDS.  Deterministic.
constexpr int kReduceWaves = 16;
constexpr int kReduceMaxLoads = 16;      // rows per half-wave: covers 2 * 16 * 16 = 512 partial rows
__global__ __launch_bounds__(64 * kReduceWaves) void layer_reduce_kernel(LayerArgs a) {
    __shared__ float red[kReduceWaves][32];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, half = lane >> 5;
    const int H = a.r.H, N = a.r.N, k = a.r.k;
    const int chunks = H >> 5;
    const int t = blockIdx.x / chunks, c0 = (blockIdx.x - t * chunks) * 32 + n;
    const int nr = k * a.nkb_r, ns = a.n_shared * a.nkb_s, nrows = nr + ns;
    const float* base_r = a.part_r + (size_t)(t * k) * a.nkb_r * H + c0;     // pairs t*k .. t*k+k-1, their blocks
    const float* base_s = a.part_s + (size_t)t * H + c0;
    float acc = 0.f;
    for (int i0 = 2 * wave + half; i0 < nrows; i0 += 2 * kReduceWaves * kReduceMaxLoads) {
        float v[kReduceMaxLoads];
#pragma unroll
        for (int j = 0; j < kReduceMaxLoads; ++j) {
            const int i = i0 + 2 * kReduceWaves * j;
            v[j] = 0.f;
            if (i < nrows) v[j] = i < nr ? base_r[(size_t)i * H] : base_s[(size_t)(i - nr) * N * H];
        }
#pragma unroll
        for (int j = 0; j < kReduceMaxLoads; ++j) acc += v[j];
    }
    acc += __shfl_xor(acc, 32, 64);
    if (half == 0) red[wave][n] = acc;
    __syncthreads();
    if (wave == 0 && half == 0) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kReduceWaves; ++w) s += red[w][n];
        if (a.y_is_fp32) static_cast<float*>(a.y)[(size_t)t * H + c0] = s;
        else static_cast<uint16_t*>(a.y)[(size_t)t * H + c0] = (uint16_t)f32_to_bf16_bits(s);
    }
}

fate_status launch_layer_decode(hipStream_t st, const fate_ffn_desc& d, LayerArgs a) {
    if (d.N < 1 || d.N > kLayerMaxN || d.N * d.k > kLayerMaxP)
        FATE_FAIL(FATE_ESHAPE, "fused layer: need 1 <= N <= %d and N*k <= %d (N = %d, k = %d)", kLayerMaxN,
                  kLayerMaxP, d.N, d.k);
    if (d.bits == 2 || (d.n_shared && d.shared_bits == 2))
        FATE_FAIL(FATE_ESHAPE, "fused layer: 4- and 8-bit experts only (2-bit copies go through fate_moe_ffn_q)");
    if (!decode_group_ok(d.bits, d.group) || (d.n_shared && !decode_group_ok(d.shared_bits, d.shared_group)))
        FATE_FAIL(FATE_ESHAPE, "fused layer: group must be 64, 128 or 256 (int4) / 64 or 128 (int8)");
    const WorkLds L = work_lds(d.N, d.H, d.E, d.k);
    constexpr int kLdsMax = 128 * 1024;
    if (L.bytes > kLdsMax) FATE_FAIL(FATE_ESHAPE, "fused layer: N = %d, H = %d need %d bytes of LDS", d.N, d.H, L.bytes);
    const int rows = (a.r.Wg2 ? 2 : 1) * d.E;
    a.nb_route = (rows + kLayerWaves - 1) / kLayerWaves;
    a.nkb_r = d.I_max / kLayerNeurons;
    a.nkb_s = d.n_shared ? d.I_shared_max / kLayerNeurons : 0;
    a.nact = min(d.E, d.N * d.k);
    {   // one token: the kernel that hands h over between workgroups instead of partial output rows
        B1Args b1;
        int nblocks = 0;
        if (b1_plan(d, a, &b1, &nblocks)) return launch_layer_decode_b1(st, d, b1, nblocks);
    }
    // work items: 32-neuron blocks of the shared experts, then of the routed slots.  With more
    // items than workgroups of the looping kernel fit on the device (asked of the occupancy
    // calculator for this launch's LDS size), the launch has that many work blocks and a block
    // takes every nwork-th item.
    static int cu_count = 0;
    if (cu_count == 0) {
        int dev = 0;
        FATE_HIP(hipGetDevice(&dev));
        FATE_HIP(hipDeviceGetAttribute(&cu_count, hipDeviceAttributeMultiprocessorCount, dev));
    }
    a.nitems = d.n_shared * a.nkb_s + a.nact * a.nkb_r;
    const int bits_s = d.n_shared ? d.shared_bits : d.bits, group_s = d.n_shared ? d.shared_group : d.group;
    const int tpg_r = d.group / (d.bits == 4 ? 64 : 32), tpg_s = group_s / (bits_s == 4 ? 64 : 32);
    int per_cu = 2;
    if (a.nitems > 2 * cu_count - a.nb_route) {
        // the query is not free: one answer per format combination and LDS size is kept
        static int key_seen[4] = {-1, -1, -1, -1}, val_seen[4] = {0, 0, 0, 0};
        const int key = ((d.bits * 8 + tpg_r) * 16 + bits_s) * 8 + tpg_s;
        int slot = -1;
        for (int i = 0; i < 4; ++i)
            if (key_seen[i] == key * 4096 + L.bytes / 64) slot = i;
        if (slot < 0) {
            int nb = 0;
#define FATE_OCC_BODY(BR, TR) nb = layer_loop_blocks_per_cu_##BR##_##TR(bits_s, tpg_s, L.bytes, kLdsMax);
            FATE_FORMAT_SWITCH(d.bits, tpg_r, FATE_OCC_BODY)
#undef FATE_OCC_BODY
            if (nb < 1) FATE_FAIL(FATE_EHIP, "fused layer: the looping kernel does not fit on a compute unit (LDS %d bytes)", L.bytes);
            static int next = 0;
            slot = next++ % 4;
            key_seen[slot] = key * 4096 + L.bytes / 64;
            val_seen[slot] = nb;
        }
        per_cu = val_seen[slot];
    }
    const int fit = std::max(1, per_cu * cu_count - a.nb_route);
    a.nwork = a.nitems > fit ? fit : a.nitems;
    const int grid = a.nb_route + a.nwork;
    fate_status rc = FATE_OK;
#define FATE_ROUTED_BODY(BR, TR)                                                                          \
    rc = a.nwork < a.nitems ? launch_layer_loop_##BR##_##TR(st, bits_s, tpg_s, grid, L.bytes, kLdsMax, a)    \
                            : launch_layer_routed<BR, TR, false>(st, bits_s, tpg_s, grid, L.bytes, kLdsMax, a);
    FATE_FORMAT_SWITCH(d.bits, tpg_r, FATE_ROUTED_BODY)
#undef FATE_ROUTED_BODY
    if (rc != FATE_OK) return rc;
    layer_reduce_kernel<<<d.N * (d.H / 32), 64 * kReduceWaves, 0, st>>>(a);
    FATE_HIP(hipGetLastError());
    return FATE_OK;
}


}  // namespace fate
