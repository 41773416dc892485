// One-token form of the one-call decode layer: arguments and the host-side plan.
//
// With one token the partial output rows of the general kernel (one row of H
// floats per 32-neuron block, summed by a second launch) are replaced by a
// hand-over of h itself, which is small: an "up" block publishes its 32 values
// of h as epoch-tagged words, a "down" block owns 32 output rows, fetches its
// slice of W2 before h exists, polls h, multiplies and writes y.  One launch,
// deterministic, no second pass over partial rows.
#pragma once
#include "layer_decode.h"

namespace fate {

constexpr int kB1MaxTiles = 24;      // W2 tiles a down wave keeps in registers
constexpr int kB1MaxItems = 64;      // wave work items of the down blocks of one output row block

// Work of one wave of a down block: `ng` quantisation groups starting at group g0 of the down
// projection of source `src` (shared expert src < n_shared, else routed slot src - n_shared).
struct B1Item {
    int16_t src, g0, ng, pad;
};

struct B1Args {
    LayerArgs a;              // its hq / yq: tagged pairs of h, tagged partial outputs
    int n_up_s, n_up_r;       // up blocks of the shared experts / of the routed slots
    int nparts, nparts_s;     // down blocks per output row block; the first nparts_s hold the shared experts' items
    int nrb;                  // output row blocks (H / 32)
    B1Item items[kB1MaxItems];
};

// true (and *b filled in, blocks counted) if the call can take the one-token path
bool b1_plan(const fate_ffn_desc& d, const LayerArgs& a, B1Args* b, int* nblocks);
fate_status launch_layer_decode_b1(hipStream_t st, const fate_ffn_desc& d, const B1Args& b, int nblocks);
// blocks of the one-token kernel that fit on the device at once (0 if it cannot run here)
int b1_resident_blocks(const fate_ffn_desc& d);

}  // namespace fate
