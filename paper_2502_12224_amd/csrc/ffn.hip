// fate_moe_ffn_q: argument checks, workspace carving, dispatch.
#include <mutex>
#include "common.h"
#include "ffn_internal.h"
#include "layer_decode.h"
#include "../../include/fate_profile.h"

namespace fate {

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static fate_status check_desc(const fate_ffn_desc* d) {
    if (d == nullptr) FATE_FAIL(FATE_EINVAL, "descriptor is NULL");
    if (d->N < 0) FATE_FAIL(FATE_EINVAL, "N = %d < 0", d->N);
    if (d->E < 1 || d->E > kMaxE) FATE_FAIL(FATE_ESHAPE, "E = %d outside [1, %d]", d->E, kMaxE);
    if (d->k < 1 || d->k > d->E) FATE_FAIL(FATE_EINVAL, "k = %d outside [1, E]", d->k);
    if (d->H < 64 || d->H % 64) FATE_FAIL(FATE_ESHAPE, "H = %d must be a positive multiple of 64", d->H);
    if (d->bits != 2 && d->bits != 4 && d->bits != 8) FATE_FAIL(FATE_EINVAL, "bits = %d (2, 4 or 8)", d->bits);
    if (d->group < 64 || d->group % 64) FATE_FAIL(FATE_ESHAPE, "group = %d must be a multiple of 64", d->group);
    if (d->I_max < 64 || d->I_max % 64) FATE_FAIL(FATE_ESHAPE, "I_max = %d must be a multiple of 64", d->I_max);
    if (d->H % d->group || d->I_max % d->group)
        FATE_FAIL(FATE_ESHAPE, "H and I_max must be multiples of the group (%d)", d->group);
    if (d->n_shared < 0 || d->n_shared > 16) FATE_FAIL(FATE_EINVAL, "n_shared = %d outside [0, 16]", d->n_shared);
    if (d->n_shared) {
        if (d->shared_bits != 2 && d->shared_bits != 4 && d->shared_bits != 8)
            FATE_FAIL(FATE_EINVAL, "shared_bits = %d", d->shared_bits);
        if (d->shared_group < 64 || d->shared_group % 64) FATE_FAIL(FATE_ESHAPE, "shared_group = %d", d->shared_group);
        if (d->I_shared_max < 64 || d->I_shared_max % 64 || d->I_shared_max % d->shared_group || d->H % d->shared_group)
            FATE_FAIL(FATE_ESHAPE, "I_shared_max = %d / H must be multiples of 64 and of the shared group", d->I_shared_max);
    }
    if (d->mode < 0 || d->mode > 2) FATE_FAIL(FATE_EINVAL, "mode = %d", d->mode);
    if (d->reserved != 0) FATE_FAIL(FATE_EINVAL, "the descriptor's reserved field must be 0");
    if ((long long)d->N * d->k > 0x3fffffffLL) FATE_FAIL(FATE_ESHAPE, "N*k too large");
    return FATE_OK;
}

static void carve(const fate_ffn_desc& d, void* base, FfnWorkspace* w) {
    char* p = static_cast<char*>(base);
    size_t off = 0;
    w->status = reinterpret_cast<int32_t*>(p + off); off += 256;
    w->h_r = reinterpret_cast<__half*>(p + off);
    off += align_up((size_t)d.N * d.k * d.I_max * 2, 256);
    w->h_s = reinterpret_cast<__half*>(p + off);
    off += align_up((size_t)d.n_shared * d.N * (d.n_shared ? d.I_shared_max : 0) * 2, 256);
    const bool mfma = d.mode == 2 || (d.mode == 0 && d.N > 16);
    w->part_r = w->part_s = reinterpret_cast<float*>(p + off);
    if (!mfma) {
        const int ncr = decode_down_chunks(d.I_max / d.group);
        const int ncs = d.n_shared ? decode_down_chunks(d.I_shared_max / d.shared_group) : 0;
        off += align_up((size_t)d.N * d.k * ncr * d.H * 4, 256);
        w->part_s = reinterpret_cast<float*>(p + off);
        off += align_up((size_t)d.n_shared * ncs * d.N * d.H * 4, 256);
    }
    if (mfma) {
        const size_t nseg1 = (size_t)d.E + d.n_shared + 1;
        w->ms.xh = reinterpret_cast<__half*>(p + off); off += align_up((size_t)d.N * d.H * 2, 256);
        w->ms.sgate = reinterpret_cast<float*>(p + off); off += align_up((size_t)d.N * 4, 256);
        w->ms.tab_up = reinterpret_cast<int32_t*>(p + off); off += align_up(nseg1 * 4, 256);
        w->ms.tab_down = reinterpret_cast<int32_t*>(p + off); off += align_up(nseg1 * 4, 256);
        w->ms.yp_r = reinterpret_cast<__half*>(p + off); off += align_up((size_t)d.N * d.k * d.H * 2, 256);
        w->ms.yp_s = reinterpret_cast<__half*>(p + off); off += align_up((size_t)d.n_shared * d.N * d.H * 2, 256);
    }
    w->bytes = off + 256;
}

}  // namespace fate

using namespace fate;

extern "C" fate_status fate_moe_ffn_q_workspace(const fate_ffn_desc* d, size_t* bytes) {
    fate_status s = check_desc(d);
    if (s != FATE_OK) return s;
    if (bytes == nullptr) FATE_FAIL(FATE_EINVAL, "bytes is NULL");
    FfnWorkspace w;
    carve(*d, nullptr, &w);
    *bytes = w.bytes;
    return FATE_OK;
}

static fate_status ffn_q_phase(int phase, const PartSel& sel, void* stream, const fate_ffn_desc* d, const void* x_bf16,
                                      const fate_qexpert* experts_dev, const int32_t* counts,
                                      const int32_t* offsets, const int32_t* perm, const int32_t* inv_perm,
                                      const int32_t* expert_order, const float* topk_w, const fate_qexpert* shared_dev,
                                      const void* shared_gate_bf16, void* y, void* workspace,
                                      size_t workspace_bytes) {
    fate_status s = check_desc(d);
    if (s != FATE_OK) return s;
    if (d->N == 0) return FATE_OK;
    FATE_CHECK_PTR(x_bf16);
    FATE_CHECK_PTR(y);
    FATE_CHECK_PTR_OPT(shared_gate_bf16);
    if (!experts_dev || !counts || !offsets || !perm || !inv_perm || !expert_order || !topk_w)
        FATE_FAIL(FATE_EINVAL, "experts, counts, offsets, perm, inv_perm, expert_order and topk_w must not be NULL");
    if (d->n_shared && !shared_dev) FATE_FAIL(FATE_EINVAL, "shared_dev is NULL with n_shared = %d", d->n_shared);
    FfnWorkspace w;
    carve(*d, workspace, &w);
    if (workspace == nullptr || workspace_bytes < w.bytes)
        FATE_FAIL(FATE_EWORKSPACE, "workspace of %zu bytes needed, %zu given", w.bytes, workspace_bytes);
    FATE_CHECK_PTR(workspace);

    DecodeArgs a{};
    a.x = static_cast<const uint16_t*>(x_bf16);
    a.N = d->N; a.H = d->H; a.E = d->E; a.k = d->k;
    a.experts = experts_dev; a.shared = shared_dev; a.n_shared = d->n_shared;
    a.counts = counts; a.offsets = offsets; a.perm = perm; a.inv_perm = inv_perm; a.order = expert_order; a.topk_w = topk_w;
    a.shared_gate = static_cast<const uint16_t*>(shared_gate_bf16);
    a.bits_r = d->bits; a.group_r = d->group;
    a.bits_s = d->n_shared ? d->shared_bits : d->bits; a.group_s = d->n_shared ? d->shared_group : d->group;
    a.h_r = w.h_r; a.ldh_r = d->I_max;
    a.h_s = w.h_s; a.ldh_s = d->n_shared ? d->I_shared_max : 0;
    a.part_r = w.part_r; a.part_s = w.part_s;
    a.status = w.status;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int mode = d->mode ? d->mode : (d->N <= 16 ? 1 : 2);
    if (mode == 1) {
        if (phase != 0 || !sel.first || !sel.last || ~sel.mask[0] || ~sel.mask[1] || ~sel.mask[2] || ~sel.mask[3])
            FATE_FAIL(FATE_EINVAL, "the decode kernels run the whole FFN only (no phases, no pieces)");
        return launch_ffn_decode(st, *d, a, y);
    }
    return launch_ffn_mfma(st, *d, a, w.ms, y, phase, sel);
}

extern "C" fate_status fate_moe_ffn_q(void* stream, const fate_ffn_desc* d, const void* x_bf16,
                                      const fate_qexpert* experts_dev, const int32_t* counts,
                                      const int32_t* offsets, const int32_t* perm, const int32_t* inv_perm,
                                      const int32_t* expert_order, const float* topk_w, const fate_qexpert* shared_dev,
                                      const void* shared_gate_bf16, void* y, void* workspace,
                                      size_t workspace_bytes) {
    return ffn_q_phase(0, part_all(), stream, d, x_bf16, experts_dev, counts, offsets, perm, inv_perm, expert_order,
                       topk_w, shared_dev, shared_gate_bf16, y, workspace, workspace_bytes);
}

extern "C" fate_status fate_moe_ffn_q_part(void* stream, const fate_ffn_desc* d, const void* x_bf16,
                                           const fate_qexpert* experts_dev, const int32_t* counts,
                                           const int32_t* offsets, const int32_t* perm, const int32_t* inv_perm,
                                           const int32_t* expert_order, const float* topk_w,
                                           const fate_qexpert* shared_dev, const void* shared_gate_bf16, void* y,
                                           void* workspace, size_t workspace_bytes, const int32_t* part_experts,
                                           int n_part, int flags) {
    if (n_part < 0 || (n_part > 0 && part_experts == nullptr) || (flags & ~3))
        FATE_FAIL(FATE_EINVAL, "fate_moe_ffn_q_part: n_part = %d, flags = %d", n_part, flags);
    PartSel sel{{0, 0, 0, 0}, (flags & 1) != 0, (flags & 2) != 0};
    for (int i = 0; i < n_part; ++i) {
        const int e = part_experts[i];
        if (d == nullptr || e < 0 || e >= d->E) FATE_FAIL(FATE_EINVAL, "part_experts[%d] = %d out of range", i, e);
        sel.mask[e >> 6] |= 1ull << (e & 63);
    }
    return ffn_q_phase(0, sel, stream, d, x_bf16, experts_dev, counts, offsets, perm, inv_perm, expert_order, topk_w,
                       shared_dev, shared_gate_bf16, y, workspace, workspace_bytes);
}

extern "C" fate_status fate_profile_ffn_mfma_phase(void* stream, const fate_ffn_desc* d, int phase,
                                                   const void* x_bf16, const fate_qexpert* experts_dev,
                                                   const int32_t* counts, const int32_t* offsets,
                                                   const int32_t* perm, const int32_t* inv_perm,
                                                   const int32_t* expert_order, const float* topk_w,
                                                   const fate_qexpert* shared_dev, const void* shared_gate_bf16,
                                                   void* y, void* workspace, size_t workspace_bytes) {
    if (phase != 1 && phase != 2) FATE_FAIL(FATE_EINVAL, "phase = %d (1 = up half, 2 = down half)", phase);
    return ffn_q_phase(phase, part_all(), stream, d, x_bf16, experts_dev, counts, offsets, perm, inv_perm, expert_order, topk_w,
                       shared_dev, shared_gate_bf16, y, workspace, workspace_bytes);
}

extern "C" fate_status fate_moe_layer_decode_workspace(const fate_ffn_desc* d, size_t* bytes,
                                                       size_t* status_offset) {
    fate_status s = check_desc(d);
    if (s != FATE_OK) return s;
    if (bytes == nullptr) FATE_FAIL(FATE_EINVAL, "bytes is NULL");
    const LayerWorkspace w = layer_workspace(*d);
    *bytes = w.bytes;
    if (status_offset) *status_offset = w.status;
    return FATE_OK;
}

namespace fate {

// Everything of fate_moe_layer_decode after the descriptor check; `status` may point outside
// the workspace.
static fate_status layer_decode_checked(void* stream, const fate_ffn_desc* d, const void* x_bf16,
                                        const void* Wg_bf16, const float* bias, const void* Wg_next_bf16,
                                        const float* bias_next, int m, int renorm, const int32_t* hint_ids,
                                        const fate_route_out* out,
                                        const fate_qexpert* experts_dev, const fate_qexpert* shared_dev,
                                        const void* shared_gate_bf16, void* y, void* workspace,
                                        size_t workspace_bytes, int32_t* status) {
    if (d->mode == 2) FATE_FAIL(FATE_EINVAL, "the fused layer call has no MFMA-GEMM mode");
    if (d->N < 1) FATE_FAIL(FATE_ESHAPE, "fused layer: N = %d < 1", d->N);
    if (m < d->k || m > d->E || m > kMaxM) FATE_FAIL(FATE_EINVAL, "need k <= m <= min(E, %d) (m = %d)", kMaxM, m);
    FATE_CHECK_PTR(x_bf16);
    FATE_CHECK_PTR(Wg_bf16);
    FATE_CHECK_PTR_OPT(bias);
    FATE_CHECK_PTR_OPT(Wg_next_bf16);
    FATE_CHECK_PTR_OPT(bias_next);
    FATE_CHECK_PTR(y);
    FATE_CHECK_PTR_OPT(shared_gate_bf16);
    if (out == nullptr || !out->topk_ids || !out->topk_w || !out->counts || !out->offsets || !out->perm ||
        !out->inv_perm || !out->expert_order)
        FATE_FAIL(FATE_EINVAL, "routing outputs must not be NULL");
    if (Wg_next_bf16 && (!out->pred_ids || !out->pred_w || !out->pred_pop))
        FATE_FAIL(FATE_EINVAL, "prediction outputs must not be NULL when the next gate is given");
    if (!experts_dev) FATE_FAIL(FATE_EINVAL, "experts_dev is NULL");
    if (d->n_shared && !shared_dev) FATE_FAIL(FATE_EINVAL, "shared_dev is NULL with n_shared = %d", d->n_shared);
    const LayerWorkspace w = layer_workspace(*d);
    if (workspace == nullptr || workspace_bytes < w.bytes)
        FATE_FAIL(FATE_EWORKSPACE, "workspace of %zu bytes needed, %zu given", w.bytes, workspace_bytes);
    FATE_CHECK_PTR(workspace);
    char* base = static_cast<char*>(workspace);

    LayerArgs a{};
    a.r = FusedRouteArgs{static_cast<const uint16_t*>(x_bf16), static_cast<const uint16_t*>(Wg_bf16), bias,
                         static_cast<const uint16_t*>(Wg_next_bf16), bias_next, d->N, d->H, d->E, d->k, m,
                         renorm != 0, out->topk_ids, out->topk_w, out->pred_ids, out->pred_w, out->pred_pop,
                         out->counts, out->offsets, out->perm, out->inv_perm, out->expert_order, nullptr};
    a.zq = reinterpret_cast<unsigned long long*>(base + w.zq);
    a.experts = experts_dev; a.shared = shared_dev; a.n_shared = d->n_shared;
    a.shared_gate = static_cast<const uint16_t*>(shared_gate_bf16);
    a.bits_r = d->bits; a.group_r = d->group;
    a.bits_s = d->n_shared ? d->shared_bits : d->bits; a.group_s = d->n_shared ? d->shared_group : d->group;
    a.part_r = reinterpret_cast<float*>(base + w.part_r);
    a.part_s = reinterpret_cast<float*>(base + w.part_s);
    a.hq = reinterpret_cast<unsigned long long*>(base + w.hq);
    a.yq = reinterpret_cast<unsigned long long*>(base + w.yq);
    a.hint = hint_ids;
    a.y = y;
    a.y_is_fp32 = d->y_is_fp32;
    a.status = status ? status : reinterpret_cast<int32_t*>(base + w.status);
    a.sync = reinterpret_cast<int32_t*>(base + w.sync);
    return launch_layer_decode(static_cast<hipStream_t>(stream), *d, a);
}

}  // namespace fate

extern "C" fate_status fate_moe_layer_decode(void* stream, const fate_ffn_desc* d, const void* x_bf16,
                                             const void* Wg_bf16, const float* bias, const void* Wg_next_bf16,
                                             const float* bias_next, int m, int renorm, const int32_t* hint_ids,
                                             const fate_route_out* out,
                                             const fate_qexpert* experts_dev, const fate_qexpert* shared_dev,
                                             const void* shared_gate_bf16, void* y, void* workspace,
                                             size_t workspace_bytes) {
    fate_status s = check_desc(d);
    if (s != FATE_OK) return s;
    return layer_decode_checked(stream, d, x_bf16, Wg_bf16, bias, Wg_next_bf16, bias_next, m, renorm, hint_ids, out,
                                experts_dev, shared_dev, shared_gate_bf16, y, workspace, workspace_bytes, nullptr);
}

// ---- the same call for callers that cannot allocate ---------------------------
// The layer kernels' workspace (epoch and exit counters, tagged logits, partial output rows)
// lives in a file-scope device array; each device holds its own copy at its own address,
// looked up once per device.  Zero-initialised when the code object is loaded, which is the
// state the kernels expect before their first call; every call leaves the counters at zero
// and overwrites the rest.
namespace fate {
constexpr size_t kScratchBytes = FATE_NOALLOC_SCRATCH_BYTES;
constexpr int kScratchMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
static void* g_scratch_ptr[kScratchMaxDevices];
static std::mutex g_scratch_mutex;

static fate_status scratch_of_current_device(void** out) {
    int dev = -1;
    FATE_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kScratchMaxDevices) FATE_FAIL(FATE_EINVAL, "device index %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        FATE_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (p == nullptr) FATE_FAIL(FATE_EHIP, "hipGetSymbolAddress returned no address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return FATE_OK;
}
}  // namespace fate

extern "C" fate_status fate_moe_layer_decode_noalloc(void* stream, const fate_ffn_desc* d, const void* x_bf16,
                                                     const void* Wg_bf16, const float* bias,
                                                     const void* Wg_next_bf16, const float* bias_next, int m,
                                                     int renorm, const int32_t* hint_ids, const fate_route_out* out,
                                                     const fate_qexpert* experts_dev, const fate_qexpert* shared_dev,
                                                     const void* shared_gate_bf16, void* y, int32_t* status_dev) {
    fate_status s = check_desc(d);
    if (s != FATE_OK) return s;
    if (status_dev == nullptr) FATE_FAIL(FATE_EINVAL, "status_dev is NULL");
    const LayerWorkspace w = layer_workspace(*d);
    if (w.bytes > kScratchBytes)
        FATE_FAIL(FATE_EWORKSPACE, "this shape needs %zu bytes of scratch, the built-in array holds %zu "
                  "(use fate_moe_layer_decode with a workspace of your own)", w.bytes, kScratchBytes);
    void* ptr = nullptr;
    s = scratch_of_current_device(&ptr);
    if (s != FATE_OK) return s;
    return layer_decode_checked(stream, d, x_bf16, Wg_bf16, bias, Wg_next_bf16, bias_next, m, renorm, hint_ids, out,
                                experts_dev, shared_dev, shared_gate_bf16, y, ptr, kScratchBytes, status_dev);
}
