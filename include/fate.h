/*
 * libfate -- MI355X (gfx950) hot path of Fate's offloaded MoE inference:
 * gate routing, cross-layer expert prediction, token-to-expert permutation,
 * grouped SwiGLU expert FFN over group-quantised weights, and the
 * shallow-favoring expert cache step.
 *
 * Conventions
 *  - Plain C ABI.  Every call returns a fate_status (0 = ok) and never throws;
 *    fate_last_error() returns a thread-local message for the last failure.
 *  - "dev" pointers are device (HBM) pointers, 16-byte aligned, owned by the
 *    caller and alive until the work enqueued on `stream` has finished.
 *    "host" pointers are ordinary host memory read during the call.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls validate their arguments, enqueue kernels and return without
 *    synchronising.  The library allocates no device memory in these calls;
 *    scratch comes in through `workspace` (size from the *_workspace query).
 *  - All tensors are row-major.  N tokens, H hidden size, E routed experts,
 *    k experts per token, I expert intermediate size, P = N*k (token, expert)
 *    pairs; pair index p = t*k + j.
 *  - Limits: 1 <= E <= 256, 1 <= k <= m <= min(E, 64), H % 64 == 0.
 */
#ifndef FATE_H
#define FATE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FATE_OK = 0,
    FATE_EINVAL = 1,       /* null pointer, value out of range */
    FATE_ESHAPE = 2,       /* shape not supported (divisibility, limits) */
    FATE_EALIGN = 3,       /* device pointer not 16-byte aligned */
    FATE_EWORKSPACE = 4,   /* workspace missing or too small */
    FATE_ENOTRESIDENT = 5, /* an activated expert has no device copy */
    FATE_EHIP = 6,         /* a HIP runtime call (or the copy callback) failed */
    FATE_ECAPACITY = 7     /* no free expert slot for a demand load */
} fate_status;

const char* fate_last_error(void);
const char* fate_version(void);

/* ------------------------------------------------------------------------
 * Gate of one MoE layer: softmax over all experts, top-k selection
 * (paper section 2.1; section 4.2 "Similar Routing Weights": the routing
 * weights over all experts sum to 1 and the k largest are selected).
 *
 *   z[t,e] = sum_h x[t,h]*Wg[e,h] + bias[e]   (fp32 accumulation)
 *   p      = softmax_e(z)
 *   ids    = the k experts with the largest z, ordered by z descending,
 *            ties to the lower id;  w = p[ids] (divided by their sum if renorm)
 *
 * x_bf16 [N,H] dev, Wg_bf16 [E,H] dev, bias [E] fp32 dev or NULL.
 * Outputs (dev): topk_ids [N,k] int32, topk_w [N,k] fp32, probs [N,E] fp32 or
 * NULL.  N == 0 is allowed (nothing is launched).
 * ---------------------------------------------------------------------- */
fate_status fate_gate_route(void* stream, const void* x_bf16, const void* Wg_bf16, const float* bias,
                            int N, int H, int E, int k, int renorm,
                            int32_t* topk_ids, float* topk_w, float* probs);

/* ------------------------------------------------------------------------
 * Cross-layer expert prediction (paper section 4.3: the gate input of block
 * i is fed to the gate of block i+1; section 4.2: widening the set beyond k
 * recovers near misses; section 4.3 "Prefill Stage": per-expert popularity
 * aggregated over tokens).
 *
 * Same arithmetic as fate_gate_route with the NEXT layer's gate on THIS
 * layer's x, width m (k <= m <= E), weights not renormalised.
 * Outputs (dev): pred_ids [N,m] int32, pred_w [N,m] fp32,
 * pred_pop [E] int32 = number of tokens whose top-m contains e (overwritten).
 * ---------------------------------------------------------------------- */
fate_status fate_cross_layer_predict(void* stream, const void* x_bf16, const void* Wg_next_bf16,
                                     const float* bias_next, int N, int H, int E, int k, int m,
                                     int32_t* pred_ids, float* pred_w, int32_t* pred_pop);

/* ------------------------------------------------------------------------
 * Token-to-expert permutation (paper section 4.3 "Prefill Stage": token-to-
 * expert assignments are aggregated and experts ranked by popularity).
 *
 * topk_ids [N,k] int32 dev, every id in [0,E).  Outputs (dev, int32):
 *   counts [E]; offsets [E+1] exclusive prefix sum (offsets[E] = N*k);
 *   perm [N*k]: pair index at sorted position s, ordered by (expert, pair);
 *   inv_perm [N*k]: its inverse;
 *   expert_order [E]: experts by (count descending, id ascending).
 * Deterministic and stable; ids outside [0,E) are not detected on the device
 * (the host cannot see them): such pairs are dropped from every output.
 * ---------------------------------------------------------------------- */
fate_status fate_permute(void* stream, const int32_t* topk_ids, int N, int k, int E,
                         int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                         int32_t* expert_order);

/* ------------------------------------------------------------------------
 * Fused routing: fate_gate_route + fate_cross_layer_predict + fate_permute
 * in one call.  N <= 16 (decode): one launch, the two gate matrices spread
 * over many compute units.  N >= 64 with H a multiple of 1024 (prefill): both
 * gate products in one launch on the matrix cores, then the permutation.
 * Other N are rejected (FATE_ESHAPE).  Same outputs, bit for bit, as the
 * three calls.  Wg_next may be NULL (last layer): pred_* are then left
 * untouched.
 * workspace: fate_route_fused_workspace bytes, zero-filled once by the
 * caller before the first use (the call leaves it zero-filled).
 * ---------------------------------------------------------------------- */
fate_status fate_route_fused_workspace(int N, int E, size_t* bytes);
fate_status fate_route_fused(void* stream, const void* x_bf16, const void* Wg_bf16, const float* bias,
                             const void* Wg_next_bf16, const float* bias_next,
                             int N, int H, int E, int k, int m, int renorm,
                             int32_t* topk_ids, float* topk_w,
                             int32_t* pred_ids, float* pred_w, int32_t* pred_pop,
                             int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                             int32_t* expert_order, void* workspace, size_t workspace_bytes);

/* ------------------------------------------------------------------------
 * Quantised expert weights.
 *
 * Canonical stored form (what a quantiser produces; paper section 4.5 stores
 * experts as low-bit integers and dequantises before compute): symmetric
 * codes q with one fp16 scale per `group` consecutive elements along the
 * reduction dimension of an output row, w = q*s; optionally one fp16
 * zero-point per group as well (see fate_qexpert), w = (u - z)*s.
 *   int8: two's-complement bytes [rows,K];  int4: nibble u = q+8, two per
 *   byte, low nibble = even column, [rows,K/2];  scales fp16 [rows,K/group].
 *   int2 (the low-precision copy of section 4.5): field u in 0..3, four per
 *   byte, column 4b+i in bits 2i..2i+1 of byte b, [rows,K/4]; the code is the
 *   odd integer q = 2u-3, i.e. the levels -3s, -s, s, 3s of the group.
 *
 * Device-native form used by the FFN kernels: 1 KiB tiles of 32 rows x
 * (128 | 64 | 32) columns (int2 | int4 | int8), one 16-byte piece per lane of a
 * wavefront, so that a wave-wide load is one contiguous KiB and each lane's
 * piece feeds its MFMA operand or its dot products directly.
 * fate_pack_weight converts canonical -> device-native (dev to dev, same
 * byte size, out of place).  rows % 32 == 0, K % 64 == 0 (K % 128 == 0 for int2).
 * Device-native scales are group-major, fp16 [K/group, rows]: the 32 rows of
 * a tile find their scales of one group in 64 contiguous bytes.
 * fate_pack_scales transposes canonical [rows, groups] into that form (dev
 * to dev, out of place).
 * ---------------------------------------------------------------------- */
fate_status fate_pack_weight(void* stream, const void* canonical_dev, int rows, int K, int bits,
                             void* packed_dev);
fate_status fate_pack_scales(void* stream, const void* canonical_dev, int rows, int groups, void* packed_dev);

/* One SwiGLU expert on the device (an element of a device-resident table). */
typedef struct {
    const void* w1; /* gate proj  [I,H] device-native codes; NULL = not resident */
    const void* w3; /* up proj    [I,H] */
    const void* w2; /* down proj  [H,I] */
    const void* s1; /* fp16 scales, group-major [H/group, I] */
    const void* s3;
    const void* s2; /* fp16 scales, group-major [I/group, H] */
    int32_t bits;   /* 2, 4 or 8: width of THIS copy */
    int32_t group;  /* multiple of 64 */
    int32_t I;      /* intermediate size, multiple of 64 */
    int32_t reserved;
    /* fp16 zero-points per group, laid out like the scales (group-major), or NULL for the symmetric
     * formats.  With zero-points w = (u - z) * s on the stored unsigned field u (the int4 nibble or the
     * int2 field; z any fp16 value, usually in [0, 2^bits - 1]): the asymmetric format of the quantiser the
     * paper uses (HQQ, section 4.5).  All three NULL or all three set; bits must be 4 or 2 (an 8-bit entry
     * with zero-points raises status bit 2 and contributes nothing).  fate_moe_ffn_q and
     * fate_moe_ffn_q_part read them in both of their modes; the one-call decode layer takes symmetric
     * entries only (others count as not resident: status bit 0). */
    const void* z1;
    const void* z3;
    const void* z2;
    int64_t reserved2;
} fate_qexpert;   /* 96 bytes */

/* ------------------------------------------------------------------------
 * Grouped SwiGLU FFN over quantised experts, dequantised in-kernel (paper
 * section 4.1 steps 5-6; expert body per section 2.1):
 *
 *   y[t] = sum_j topk_w[t,j] * W2_e (silu(W1_e x[t]) * (W3_e x[t])), e = ids[t,j]
 *        + sum_s g_s(t) * W2_s (silu(W1_s x[t]) * (W3_s x[t]))   shared experts
 *   g_s(t) = 1, or sigmoid(x[t] . shared_gate) when shared_gate != NULL.
 *
 * x_bf16 [N,H] dev.  experts_dev: device array [E] of fate_qexpert; shared_dev:
 * device array [n_shared] or NULL.  counts/offsets/perm: outputs of
 * fate_permute for this layer's ids (dev), as are inv_perm and expert_order.
 * topk_w [N,k] dev.
 * expert_order [E] dev (from fate_permute).  y [N,H] dev, fp32 (y_is_fp32) or
 * bf16, overwritten.  I_max / I_shared_max bound the intermediate sizes in the
 * tables (host-known; used to size launches and scratch); bits/group of the
 * routed experts and of the shared experts are passed host-side as well: they
 * are the nominal format of the layer.  The kernels read the width and group of
 * every entry from the table, so a layer may mix copies of different widths
 * (the popularity-aware hybrid of section 4.5: the least popular experts of a
 * prefill arrive as 2-bit copies); a group is a whole number of tile columns
 * (128 / 64 / 32 for int2 / int4 / int8); the decode kernels take groups of
 * 64..256 columns (int4), 64 / 128 (int8), 128 / 256 (int2).
 * mode: 0 = choose (decode kernels if N <= 16, else MFMA), 1 = decode
 * dequant-GEMV kernels, 2 = MFMA grouped GEMM (H and the intermediate sizes
 * multiples of 128; N*H, N*k*I_max and n_shared*N*I_shared_max below 2^31;
 * FATE_ESHAPE otherwise).
 * Activated experts whose w1 is NULL are skipped and flagged in the int32 at
 * workspace offset 0 (bit 0); an entry whose width / group the kernels cannot
 * read is skipped too (bit 2).
 * ---------------------------------------------------------------------- */
typedef struct {
    int32_t N, H, E, k;
    int32_t I_max, bits, group;                      /* routed experts */
    int32_t n_shared, I_shared_max, shared_bits, shared_group;
    int32_t y_is_fp32;
    int32_t mode;
    int32_t reserved; /* must be 0 */
} fate_ffn_desc;

fate_status fate_moe_ffn_q_workspace(const fate_ffn_desc* d, size_t* bytes);
fate_status fate_moe_ffn_q(void* stream, const fate_ffn_desc* d, const void* x_bf16,
                           const fate_qexpert* experts_dev, const int32_t* counts, const int32_t* offsets,
                           const int32_t* perm, const int32_t* inv_perm, const int32_t* expert_order,
                           const float* topk_w,
                           const fate_qexpert* shared_dev, const void* shared_gate_bf16,
                           void* y, void* workspace, size_t workspace_bytes);

/* ------------------------------------------------------------------------
 * The same FFN taken in pieces, for a prefill layer whose experts are still
 * arriving (paper section 4.3, figure "rearranging the order of expert
 * computations": experts already on the device are computed first, the others
 * in the order of their transfers, so that computation and transfers overlap).
 * Matrix-core mode only.  Each call processes the routed experts listed in
 * part_experts (host array of n_part ids in [0,E), read during the call); a
 * caller walks through the cache step's compute_order and makes the stream wait
 * for a piece's transfers before the piece's call.
 *   flags bit 0: first piece - prepares x, and processes the shared experts;
 *   flags bit 1: last piece - adds up y (y is undefined before it).
 * Every activated expert must belong to exactly one piece; the pieces of a
 * layer share workspace and arguments and are ordered on one stream.  The
 * result equals fate_moe_ffn_q's bit for bit.
 * ---------------------------------------------------------------------- */
fate_status fate_moe_ffn_q_part(void* stream, const fate_ffn_desc* d, const void* x_bf16,
                                const fate_qexpert* experts_dev, const int32_t* counts, const int32_t* offsets,
                                const int32_t* perm, const int32_t* inv_perm, const int32_t* expert_order,
                                const float* topk_w,
                                const fate_qexpert* shared_dev, const void* shared_gate_bf16,
                                void* y, void* workspace, size_t workspace_bytes,
                                const int32_t* part_experts, int n_part, int flags);

/* ------------------------------------------------------------------------
 * Whole decode-side MoE layer in one call (1 <= N <= 8, N*k <= 64; two
 * launches: the layer kernel and a small reduction): fate_gate_route +
 * fate_cross_layer_predict + fate_permute + fate_moe_ffn_q (section 4.1
 * steps 1-2, 5-6 of one layer), with the same results as those calls:
 * routing outputs bit for bit, y up to the order of its fp32 additions.  The
 * weight stream of the shared experts starts while the gate is still being
 * evaluated; a work group owns 32 intermediate neurons of one expert, does
 * their up projection and multiplies the result into its columns of the down
 * projection, and leaves a partial output row that the reduction adds up.
 * A call with more such items than work groups fit on the device at once
 * launches as many as fit, and each takes every n-th item.
 *   hint_ids: NULL, or a device array of k expert ids predicted for THIS layer
 *        by the previous layer's call (the first k entries of its pred_ids; for
 *        N == 1 only, ignored otherwise).  A prefetch hint in the sense of
 *        section 4.3: the work groups of routed slot j start fetching expert
 *        hint_ids[j] before this layer's gate is known and keep it if the gate
 *        selects it; a wrong, repeated or out-of-range id only costs time.  The
 *        results do not depend on the hint except for the order of the fp32
 *        additions in y.
 *   out: device pointers for every routing output, sized as in the separate
 *        calls; pred_* may be NULL when Wg_next is NULL (last layer).
 *   d->mode must be 0 or 1.
 *   workspace: fate_moe_layer_decode_workspace bytes, 256-byte aligned,
 *        zero-filled once by the caller before the first use (each call
 *        leaves its counters at zero).  Calls that share a workspace must be
 *        ordered on one stream.  The int32 at byte *status_offset of the
 *        workspace is the status word: bit 0 = an activated expert had NULL
 *        weights, bit 1 = a wait inside the kernel ran out (results invalid).
 * ---------------------------------------------------------------------- */
typedef struct {
    int32_t* topk_ids; float* topk_w;
    int32_t* pred_ids; float* pred_w; int32_t* pred_pop;
    int32_t* counts; int32_t* offsets; int32_t* perm; int32_t* inv_perm; int32_t* expert_order;
} fate_route_out;

fate_status fate_moe_layer_decode_workspace(const fate_ffn_desc* d, size_t* bytes, size_t* status_offset);
fate_status fate_moe_layer_decode(void* stream, const fate_ffn_desc* d, const void* x_bf16,
                                  const void* Wg_bf16, const float* bias,
                                  const void* Wg_next_bf16, const float* bias_next, int m, int renorm,
                                  const int32_t* hint_ids, const fate_route_out* out,
                                  const fate_qexpert* experts_dev, const fate_qexpert* shared_dev,
                                  const void* shared_gate_bf16, void* y, void* workspace, size_t workspace_bytes);

/* ------------------------------------------------------------------------
 * fate_moe_layer_decode for callers that cannot allocate device memory or
 * bring a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Same arguments, kernels and results as
 * fate_moe_layer_decode, except that the kernels' workspace (call epoch and
 * exit counter, tagged logits, partial output rows) is a device array built
 * into the library, FATE_NOALLOC_SCRATCH_BYTES long, one copy per GPU, held
 * until the process ends; the call allocates nothing and calls no allocating
 * routine.  A shape whose workspace (fate_moe_layer_decode_workspace) exceeds
 * that size is rejected with FATE_EWORKSPACE.
 *   status_dev: device int32 owned by the caller, 16-byte aligned; the kernels
 *        OR the status bits of fate_moe_layer_decode into it (bit 0: an
 *        activated expert had NULL weights, bit 1: a wait ran out) and never
 *        clear it.
 * All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams, or a graph replayed while another call runs)
 * race and give wrong results; order them on one stream.
 * ---------------------------------------------------------------------- */
#define FATE_NOALLOC_SCRATCH_BYTES (32u << 20)
fate_status fate_moe_layer_decode_noalloc(void* stream, const fate_ffn_desc* d, const void* x_bf16,
                                          const void* Wg_bf16, const float* bias,
                                          const void* Wg_next_bf16, const float* bias_next, int m, int renorm,
                                          const int32_t* hint_ids, const fate_route_out* out,
                                          const fate_qexpert* experts_dev, const fate_qexpert* shared_dev,
                                          const void* shared_gate_bf16, void* y, int32_t* status_dev);

/* ------------------------------------------------------------------------
 * Expert cache (paper section 4.4: memory budget -> cache_total; boundary L;
 * shallow layers cached fully, the rest split evenly over deep layers; ARC
 * per layer.  Section 4.1 steps 3-4, 7-8: residency check, transfer of
 * predicted experts, cache-list update from the true gate result, eviction.
 * Section 4.3: transfers in descending popularity, at most n per layer;
 * compute order "on the device first, then in load order").
 *
 * The policy is host integer logic and runs without a GPU; data movement
 * goes through a copy callback.  fate_cache_create_hip installs the built-in
 * engine: hipMemcpyAsync from a pinned host pool into device slots on a side
 * stream, one event per slot, and it keeps a device table of fate_qexpert
 * per layer up to date.
 * ---------------------------------------------------------------------- */
typedef struct fate_cache fate_cache;

/* copy callback: bring the `bits`-wide copy of expert `e` of `layer` into
 * `slot`.  demand != 0 for a load the current layer waits on.  Return 0 on
 * success. */
typedef int (*fate_copy_fn)(void* user, int layer, int expert, int slot, int demand, int bits);

/* closed forms of section 4.3 / 4.4 */
int64_t fate_cache_total_from_budget(int64_t memory_budget, int64_t others, int64_t expert_bytes);
int32_t fate_n_max_from_times(double t_moe, double t_attn, double t_gate, double t_expert);
fate_status fate_cache_layer_capacities(int num_layers, int E, int cache_total, int L_shallow,
                                        int32_t* caps /*[num_layers] host out*/);

fate_cache* fate_cache_create(int num_layers, int E, int cache_total, int L_shallow, int n_max,
                              int staging_slots, fate_copy_fn copy, void* user);
void fate_cache_destroy(fate_cache*);
int32_t fate_cache_total_slots(const fate_cache*);
/* Changes the cap on prefetched experts per layer (section 4.3: n = floor(T / t_expert)); the
 * ratio differs between prefill and decode, so a caller re-calibrates between the phases.
 * n_max < 0 -> FATE_EINVAL. */
fate_status fate_cache_set_n_max(fate_cache*, int n_max);
/* Popularity-aware hybrid width of the transfers (section 4.5, "Quantization for I/O": in prefill the
 * least popular experts are moved at a lower width; the prefetch list carries the width, section 4.1
 * step 2).  Of the experts predicted for the next layer (popularity > 0), ranked by predicted
 * popularity, the last floor(percent * n / 100) are transferred as `low_bits` copies if they need a
 * transfer at all; everything else, and every demand load, moves at `bits`.  A low-width copy serves
 * its layer's computation and is then dropped: it never enters the layer's cache, which holds
 * `bits` copies only.  percent = 0 (the default) switches the rule off; a caller sets it for the
 * prefill pass and clears it for decoding, where every selected expert counts the same. */
fate_status fate_cache_set_low_precision(fate_cache*, int percent, int bits, int low_bits);
/* slot of (layer, expert) or -1; resident: 2 = in the layer's cache, 1 = staged, 0 = absent */
int32_t fate_cache_slot_of(const fate_cache*, int layer, int expert);
int32_t fate_cache_resident(const fate_cache*, int layer, int expert);

typedef struct {
    int32_t n_hit_cache, n_hit_prefetch, n_miss;   /* unique activated experts of this step */
    int32_t pair_hits, pair_misses;                /* weighted by pair counts */
    int32_t n_prefetch_issued, n_prefetch_dropped, n_wasted, n_evicted;
    int32_t n_loads;                               /* entries written to loads[] */
} fate_cache_stats;

typedef struct { int32_t layer, expert, slot, demand, bits; } fate_cache_load;

/* One cache step for `layer` (host arrays):
 *   actual_ids/actual_counts [n_actual]: unique experts the true gate chose,
 *     with their pair counts; processed in stable order of count descending.
 *   pred_ids/pred_pop [n_pred]: prediction for layer+1 (unique ids with
 *     popularity); taken in stable order of popularity descending; ignored
 *     for the last layer.
 * Outputs (host): compute_order [n_actual] (cached experts, then prefetched,
 * then demand-loaded in load order); slots [n_actual] slot of each expert in
 * compute_order; loads [max_loads] issue-ordered list of copies (demand loads
 * first, then prefetches); stats.  Slots freed in a step become reusable in
 * the next one.  Errors: FATE_ECAPACITY (no slot for a demand load),
 * FATE_EHIP (copy callback failed; the expert is not marked resident).
 */
fate_status fate_expert_cache_step(fate_cache*, int layer,
                                   const int32_t* actual_ids, const int32_t* actual_counts, int n_actual,
                                   const int32_t* pred_ids, const int32_t* pred_pop, int n_pred,
                                   int32_t* compute_order, int32_t* slots,
                                   fate_cache_load* loads, int max_loads, fate_cache_stats* stats);

/* Dense front ends.  counts [E] and pred_pop [E] (may be NULL) are the arrays
 * fate_permute / fate_cross_layer_predict produce, copied to the host; experts
 * are taken in id order (so ties in count or popularity go to the lower id).
 * compute_order / slots: host arrays of E entries; n_actual_out may be NULL. */
fate_status fate_expert_cache_step_dense(fate_cache*, int layer, const int32_t* counts, const int32_t* pred_pop,
                                         int32_t* compute_order, int32_t* slots, int32_t* n_actual_out,
                                         fate_cache_load* loads, int max_loads, fate_cache_stats* stats);
/* Accounting over a range of fully cached layers [layer_begin, layer_end):
 * counts / pred_pop are [layers][E]; the statistics are summed.  Returns
 * FATE_ENOTRESIDENT if a layer of the range is not fully cached (such layers
 * need their own step before their FFN runs). */
fate_status fate_expert_cache_step_layers(fate_cache*, int layer_begin, int layer_end, const int32_t* counts,
                                          const int32_t* pred_pop, fate_cache_stats* stats_sum);

/* ------------------------------------------------------------------------
 * Activation-path predictor: the prefetch policy of the paper's EAP baseline
 * (section 5.1: the experts of the next block are predicted from the token's
 * expert choices in the previous block and statistics collected beforehand),
 * kept as a comparison mode; its output feeds the same cache step.  Host
 * integer logic.
 *   fate_eap_update: adds one calibration batch: ids_l / ids_next [N,k] host,
 *     the choices of the same tokens in blocks `layer` and `layer`+1.
 *   fate_eap_predict: pred_pop [E] host out = number of tokens of ids_l [N,k]
 *     whose m highest positive co-activation scores include the expert (ties to
 *     the lower id); all zero for the last block.
 * ---------------------------------------------------------------------- */
typedef struct fate_eap fate_eap;
fate_eap* fate_eap_create(int num_layers, int E);
void fate_eap_destroy(fate_eap*);
fate_status fate_eap_update(fate_eap*, int layer, const int32_t* ids_l, const int32_t* ids_next, int N, int k);
fate_status fate_eap_predict(const fate_eap*, int layer, const int32_t* ids_l, int N, int k, int m,
                             int32_t* pred_pop);

/* Built-in HIP copy engine.  slot_pool_dev: total_slots * slot_bytes of device
 * memory; host_pool_pinned: num_layers*E experts of slot_bytes each (pinned),
 * expert (l,e) at ((l*E)+e)*slot_bytes, already in device-native layout with
 * the six arrays at the offsets given in `layout`.  table_dev: device array
 * [num_layers*E] of fate_qexpert maintained by the engine.  The engine enqueues
 * copies in turn on copy_stream and on a second stream of its own (default
 * priority; destroyed, after a synchronise, by fate_hip_engine_destroy), makes
 * compute_stream wait for the copies the current layer needs, and makes both
 * copy streams wait for `compute_done_event` (recorded by the caller after the
 * previous layer's FFN) before overwriting slots.  Whoever needs every copy to
 * have finished waits for the device, not for copy_stream alone. */
typedef struct {
    size_t slot_bytes;
    size_t off_w1, off_w3, off_w2, off_s1, off_s3, off_s2;
    int32_t bits, group, I;
} fate_slot_layout;

typedef struct fate_hip_engine fate_hip_engine;
fate_hip_engine* fate_hip_engine_create(int num_layers, int E, int total_slots, const fate_slot_layout* layout,
                                        void* slot_pool_dev, const void* host_pool_pinned,
                                        fate_qexpert* table_dev, void* copy_stream, void* compute_stream);
void fate_hip_engine_destroy(fate_hip_engine*);
/* the fate_copy_fn to pass to fate_cache_create together with the engine as `user` */
int fate_hip_engine_copy(void* engine, int layer, int expert, int slot, int demand, int bits);
/* Second host pool with the low-width copies (section 4.5: both widths of every expert are kept in
 * host memory): num_layers*E experts of layout->slot_bytes each, pinned, expert (l,e) at
 * ((l*E)+e)*slot_bytes.  A copy whose `bits` equals layout->bits comes from this pool and writes a
 * table entry of that width; slot_bytes must not exceed the main layout's. */
fate_status fate_hip_engine_set_low_pool(fate_hip_engine*, const fate_slot_layout* layout,
                                         const void* host_pool_low_pinned);
/* call before each fate_expert_cache_step: orders later copies after `compute_done_event` (may be NULL) */
fate_status fate_hip_engine_begin_step(fate_hip_engine*, void* compute_done_event);
/* call after the step: compute_stream waits for the copies of `layer`'s activated experts */
fate_status fate_hip_engine_wait_ready(fate_hip_engine*, const int32_t* slots, int n);
/* mark preloaded experts: write the table entry of (layer, expert) for `slot` and copy it synchronously */
fate_status fate_hip_engine_preload(fate_hip_engine*, int layer, int expert, int slot);
uint64_t fate_hip_engine_bytes_copied(const fate_hip_engine*);

#ifdef __cplusplus
}
#endif
#endif /* FATE_H */
