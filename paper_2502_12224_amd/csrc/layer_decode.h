// Whole decode-side MoE layer in one launch: arguments and workspace layout
// shared between the entry point and the kernel's translation unit.
#pragma once
#include "common.h"
#include "route_device.h"

namespace fate {

constexpr int kLayerWaves = 4;                  // waves per workgroup
constexpr int kLayerThreads = 64 * kLayerWaves;
constexpr int kLayerNeurons = 32;               // intermediate neurons per work block
constexpr int kLayerMaxN = 8;                   // tokens per call
constexpr int kLayerMaxP = 64;                  // (token, expert) pairs per call
constexpr int kLayerMaxParts = 16;              // one-token kernel: down blocks per output row block

struct LayerArgs {
    FusedRouteArgs r;              // x, gates, sizes, routing outputs (its zbuf is not used)
    unsigned long long* zq;        // [2][N][E] logits, each tagged with the call's epoch in the high word
    const fate_qexpert* experts;
    const fate_qexpert* shared;
    const uint16_t* shared_gate;
    int n_shared, bits_r, group_r, bits_s, group_s;
    int nb_route;                  // routing workgroups (block ids [0, nb_route))
    int nkb_r, nkb_s;              // 32-neuron blocks per routed / shared expert
    int nact;                      // routed expert slots: min(E, N*k)
    float* part_r;                 // [N*k pairs][nkb_r][H] weighted partial outputs of the routed blocks
    float* part_s;                 // [n_shared][nkb_s][N][H] same for the shared experts
    void* y;                       // [N,H] fp32 or bf16, written by the reduction kernel
    int y_is_fp32;
    int32_t* status;
    int32_t* sync;                 // [0] epoch of the previous call, [1] workgroups that have left
    const int32_t* hint;           // one-token kernel: k expert ids predicted for this layer, or NULL
    unsigned long long* hq;        // one-token kernel: tagged pairs of h, shared experts [n_shared][I_s_max / 2] then routed slots [k][I_max / 2]
    unsigned long long* yq;        // one-token kernel: [parts - 1][H] tagged partial outputs
    int nitems, nwork;             // work items (32-neuron blocks of shared experts, then of routed slots); work blocks in the launch
};

// byte offsets inside the workspace of fate_moe_layer_decode
struct LayerWorkspace {
    size_t sync, zq, status, part_r, part_s, hq, yq, bytes;
};

inline LayerWorkspace layer_workspace(const fate_ffn_desc& d) {
    const int N = d.N, H = d.H, E = d.E;
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    LayerWorkspace w;
    size_t off = 0;
    w.sync = off; off += 256;
    w.zq = off; off += up((size_t)2 * N * E * sizeof(unsigned long long));
    w.status = off; off += 256;
    w.part_r = off; off += up((size_t)N * d.k * (d.I_max / kLayerNeurons) * H * sizeof(float));
    w.part_s = off;
    off += up((size_t)d.n_shared * (d.n_shared ? d.I_shared_max / kLayerNeurons : 0) * N * H * sizeof(float));
    // one-token kernel: h words and partial outputs of up to kLayerMaxParts down blocks per row block
    w.hq = off;
    off += N == 1 ? up(((size_t)d.n_shared * (d.n_shared ? d.I_shared_max : 0) + (size_t)d.k * d.I_max) / 2 * 8) : 0;
    w.yq = off;
    off += N == 1 ? up((size_t)kLayerMaxParts * H * 8) : 0;
    w.bytes = off;
    return w;
}

fate_status launch_layer_decode(hipStream_t st, const fate_ffn_desc& d, LayerArgs a);

}  // namespace fate
