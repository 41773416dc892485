/*
 * libfate -- measurement aid, not part of the hot path.
 *
 * The prefill-side expert FFN (fate_moe_ffn_q in its matrix-core mode) is four
 * launches: preparation + the up/gate grouped GEMM with the SwiGLU epilogue
 * (paper section 2.1, the first two projections of an expert), then the down
 * grouped GEMM + the per-token combination.  A benchmark that reports the
 * matrix-core rate of the dominant GEMM times the first half alone.
 */
#ifndef FATE_PROFILE_H
#define FATE_PROFILE_H

#include "fate.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Same arguments as fate_moe_ffn_q plus `phase`: 1 = preparation and up/gate
 * GEMM only (h is left in the workspace, y untouched), 2 = down GEMM and
 * combination only (reads the h a phase-1 call left in the same workspace).
 * Matrix-core mode only: d->mode == 2, or 0 with N > 16; other calls and
 * other phase values return FATE_EINVAL. */
fate_status fate_profile_ffn_mfma_phase(void* stream, const fate_ffn_desc* d, int phase, const void* x_bf16,
                                        const fate_qexpert* experts_dev, const int32_t* counts,
                                        const int32_t* offsets, const int32_t* perm, const int32_t* inv_perm,
                                        const int32_t* expert_order, const float* topk_w,
                                        const fate_qexpert* shared_dev, const void* shared_gate_bf16, void* y,
                                        void* workspace, size_t workspace_bytes);

#ifdef __cplusplus
}
#endif
#endif /* FATE_PROFILE_H */
