// One-call decode layer: the looping kernels (several work items per block) whose routed experts
// are int4 with 1 tile(s) per group.
#include "layer_decode_impl.h"

namespace fate {

fate_status launch_layer_loop_4_1(hipStream_t st, int bits_s, int tpg_s, int grid, int lds_bytes, int lds_max,
                                   const LayerArgs& a) {
    return launch_layer_routed<4, 1, true>(st, bits_s, tpg_s, grid, lds_bytes, lds_max, a);
}

int layer_loop_blocks_per_cu_4_1(int bits_s, int tpg_s, int lds_bytes, int lds_max) {
    return layer_routed_blocks_per_cu<4, 1, true>(bits_s, tpg_s, lds_bytes, lds_max);
}

}  // namespace fate
