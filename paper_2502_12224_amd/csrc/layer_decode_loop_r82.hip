// One-call decode layer: the looping kernels (several work items per block) whose routed experts
// are int8 with 2 tile(s) per group.
#include "layer_decode_impl.h"

namespace fate {

fate_status launch_layer_loop_8_2(hipStream_t st, int bits_s, int tpg_s, int grid, int lds_bytes, int lds_max,
                                   const LayerArgs& a) {
    return launch_layer_routed<8, 2, true>(st, bits_s, tpg_s, grid, lds_bytes, lds_max, a);
}

int layer_loop_blocks_per_cu_8_2(int bits_s, int tpg_s, int lds_bytes, int lds_max) {
    return layer_routed_blocks_per_cu<8, 2, true>(bits_s, tpg_s, lds_bytes, lds_max);
}

}  // namespace fate
