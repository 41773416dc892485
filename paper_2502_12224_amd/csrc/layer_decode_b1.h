// One-token form of the one-call decode layer: arguments and the host-side plan.
//
// With one token the partial output rows of the general kernel (one row of H
// floats per 32-neuron block, summed by a second launch) are replaced by a
// hand-over of h itself, which is small: an "up" block publishes its 32 values
// of h as epoch-tagged words, a "down" block owns 32 output rows, fetches its
// slices of W2 before h exists, polls h, multiplies and writes y.  One launch,
// deterministic, no second pass over partial rows.  Every down wave holds one
// piece of the shared experts' W2 and one piece of a routed slot's: the shared
// piece is multiplied while the routed experts are still being fetched, so
// that only half of a wave's products are left once the routed h exists.
#pragma once
#include "layer_decode.h"

namespace fate {

constexpr int kB1MaxTiles = 12;      // W2 tiles per piece: a down wave keeps two pieces (shared, routed) in registers
constexpr int kB1MaxItems = 32;      // pieces of each kind over the down blocks of one output row block

// One piece of the work of a down wave: `ng` quantisation groups starting at group g0 of the down
// projection of source `src` (a shared expert for a piece of the first list, a routed slot for one
// of the second).  Wave w of down block `part` of a row block takes piece part * 4 + w of each list.
struct B1Item {
    int16_t src, g0, ng, pad;
};

struct B1Args {
    LayerArgs a;              // its hq / yq: tagged pairs of h, tagged partial outputs
    int n_up_s, n_up_r;       // up blocks of the shared experts / of the routed slots
    int nparts;               // down blocks per output row block
    int nrb;                  // output row blocks (H / 32)
    B1Item items_s[kB1MaxItems], items_r[kB1MaxItems];
};

// true (and *b filled in, blocks counted) if the call can take the one-token path
bool b1_plan(const fate_ffn_desc& d, const LayerArgs& a, B1Args* b, int* nblocks);
fate_status launch_layer_decode_b1(hipStream_t st, const fate_ffn_desc& d, const B1Args& b, int nblocks);
// blocks of the one-token kernel that fit on the device at once (0 if it cannot run here)
int b1_resident_blocks(const fate_ffn_desc& d);

}  // namespace fate
