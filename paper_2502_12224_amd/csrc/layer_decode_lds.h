// LDS layout of a work block of the one-call decode layer, shared by the kernel and by the
// host code that sizes the launch.
#pragma once
#include "common.h"
#include "decode_device.h"
#include "layer_decode.h"

namespace fate {

constexpr int kHsLd = kLayerNeurons + kLdsPad;   // halves per row of h in LDS
constexpr int kSlotWords = 2 + 3 * kTokPass;     // per routed slot: expert, row count, then token / pair / weight of each row

// LDS carve of a work block (bytes from the start of dynamic shared memory)
struct WorkLds {
    int xs, hs, red, tab, zl, ids, w, pairq, tokid, wtok, cx, ch, slots, bytes;
};
__host__ __device__ inline WorkLds work_lds(int N, int H, int E, int k) {
    auto up = [](int v) { return (v + 15) & ~15; };
    const int ntp = N < kTokPass ? N : kTokPass;
    const int P = N * k;
    WorkLds L;
    int off = 0;
    L.xs = off; off += up((N + 1) * (H + kLdsPad) * 2);
    L.hs = off; off += up((kTokPass + 1) * kHsLd * 2);
    L.red = off; off += up(kLayerWaves * 2 * ntp * 32 * 4);
    L.tab = off; off += up(E * (int)sizeof(fate_qexpert));
    L.zl = off; off += up(2 * N * E * 4);
    L.ids = off; off += up(P * 4);
    L.w = off; off += up(P * 4);
    L.pairq = off; off += up(kTokPass * 4);
    L.tokid = off; off += up(kTokPass * 4);
    L.wtok = off; off += up(kTokPass * 4);
    L.cx = off; off += up((H / 64) * (kTokPass + 1) * 4);     // [group][token] bias sums of x (groups of >= 64 columns)
    L.ch = off; off += up(kTokPass * 4);                      // [row] bias sum of h
    L.slots = off; off += up(kLayerMaxP * kSlotWords * 4);    // looping kernels: per routed slot its expert and rows
    L.bytes = off;
    return L;
}

}  // namespace fate
