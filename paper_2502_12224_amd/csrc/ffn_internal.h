// Shared between the FFN translation units.
#pragma once
#include <hip/hip_fp16.h>
#include "common.h"

namespace fate {

struct DecodeArgs {
    const uint16_t* x;
    int N, H, E, k;
    const fate_qexpert* experts;
    const fate_qexpert* shared;
    int n_shared;
    const int32_t* counts;
    const int32_t* offsets;
    const int32_t* perm;
    const int32_t* inv_perm;
    const int32_t* order;
    const float* topk_w;
    const uint16_t* shared_gate;
    int nact;            // routed expert slots in the grid: min(E, N*k)
    int rb_r, rb_s;      // 32-row blocks per routed / shared expert (up kernel)
    int bits_r, group_r, bits_s, group_s;
    __half* h_r; int ldh_r;   // [P][I_max] fp16, rows in sorted pair order
    __half* h_s; int ldh_s;   // [n_shared*N][I_shared_max] fp16
    float* part_r;            // [P][nchunk_r][H] fp32: weighted partial outputs, rows in sorted pair order
    float* part_s;            // [n_shared][nchunk_s][N][H] fp32 (gated)
    int32_t* status;
    int nchunk_r, nchunk_s, cg_r, cg_s;   // reduction chunks of the down kernel
    int lds_rows;        // activation rows staged in LDS per pass, plus one zero row
};

struct MfmaScratch {
    __half* xh;        // [N,H] fp16 copy of x
    float* sgate;      // [N] shared gate values
    int32_t* tab_up;   // [E + n_shared + 1] tile prefix sums of the up GEMM
    int32_t* tab_down; // same for the down GEMM
    __half* yp_r;      // [P,H] per-pair outputs of the down GEMM
    __half* yp_s;      // [n_shared*N,H]
};

struct FfnWorkspace {
    int32_t* status;
    __half* h_r;
    __half* h_s;
    float* part_r;   // decode path: partial outputs of the down kernel, summed in a fixed order by a last launch
    float* part_s;
    MfmaScratch ms;  // MFMA path only
    size_t bytes;
};

fate_status launch_ffn_decode(hipStream_t st, const fate_ffn_desc& d, DecodeArgs a, void* y_out);
// reduction chunks (of at most 16 groups) of the decode down kernel for an intermediate size of G groups
inline int decode_down_chunks(int G) { return G > 0 ? (G + 15) / 16 : 1; }
// Piece of a layer (matrix-core path): the routed experts of `mask` (bit e), the shared experts and
// the preparation of x with the first piece, the per-token combination with the last one.
struct PartSel {
    unsigned long long mask[4];
    int first, last;
};
inline PartSel part_all() { return PartSel{{~0ull, ~0ull, ~0ull, ~0ull}, 1, 1}; }

// phase: 0 = whole FFN, 1 = prep + up/gate GEMM only, 2 = down GEMM + combine only (timing aid)
fate_status launch_ffn_mfma(hipStream_t st, const fate_ffn_desc& d, DecodeArgs a, const MfmaScratch& ms,
                            void* y_out, int phase, const PartSel& sel);

}  // namespace fate
