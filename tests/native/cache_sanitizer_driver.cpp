// Driver for the sanitizer build of the cache policy (host-only C++): random traces through every
// mode of the cache step - plain, no cache / no prefetch, hybrid width, changing prefetch cap - and
// through the co-activation predictor.  It checks nothing about values (the Python tests compare the
// library with the oracle); it exists so that the address and undefined-behaviour sanitizers see the
// code run.  Built and run by tests/test_abi_cpu.py.
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/fate.h"

namespace fate {
void set_error(const char* fmt, ...) {      // (lives in api.cpp in the library)
    va_list ap;
    va_start(ap, fmt);
    vfprintf(stderr, fmt, ap);
    va_end(ap);
    fputc('\n', stderr);
}
}  // namespace fate

static uint32_t rng_state = 12345u;
static uint32_t rnd() {
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}

static int copy_cb(void* user, int, int, int, int, int) {
    ++*static_cast<long*>(user);
    return 0;
}

static int run_cache(int layers, int E, int cache_total, int L_shallow, int n_max, int staging, int percent, int steps) {
    long copies = 0;
    fate_cache* c = fate_cache_create(layers, E, cache_total, L_shallow, n_max, staging, copy_cb, &copies);
    if (!c) return 1;
    if (fate_cache_set_low_precision(c, percent, 4, 2) != FATE_OK) return 2;
    std::vector<int32_t> counts(E), pop(E), order(E), slots(E);
    std::vector<fate_cache_load> loads(4 * E + 8);
    fate_cache_stats st;
    for (int s = 0; s < steps; ++s) {
        if (s == steps / 2 && fate_cache_set_n_max(c, n_max / 2) != FATE_OK) return 3;
        for (int l = 0; l < layers; ++l) {
            for (int e = 0; e < E; ++e) {
                counts[e] = (rnd() % 4 == 0) ? 1 + (int)(rnd() % 5) : 0;
                pop[e] = (rnd() % 3 == 0) ? 1 + (int)(rnd() % 7) : 0;
            }
            counts[rnd() % E] = 3;
            int32_t n_act = 0;
            const fate_status rc = fate_expert_cache_step_dense(c, l, counts.data(), l + 1 < layers ? pop.data() : nullptr,
                                                                order.data(), slots.data(), &n_act, loads.data(),
                                                                (int)loads.size(), &st);
            if (rc != FATE_OK) return 4;
            for (int i = 0; i < n_act; ++i)
                if (order[i] < 0 || order[i] >= E || slots[i] < 0 || slots[i] >= fate_cache_total_slots(c)) return 5;
        }
    }
    fate_cache_destroy(c);
    return 0;
}

int main() {
    const int E = 16, layers = 5;
    int rc;
    // the method: shallow-favoring capacities, ARC in the deep layers, prefetch cap 3
    if ((rc = run_cache(layers, E, 40, 2, 3, 2 * E + 3, 0, 60))) return 10 + rc;
    // hybrid width in the prefetch list
    if ((rc = run_cache(layers, E, 40, 2, E, 2 * E + E, 25, 40))) return 20 + rc;
    // no cache, no prefetch (load on demand)
    if ((rc = run_cache(layers, E, 0, 0, 0, 2 * E, 0, 30))) return 30 + rc;
    // everything cached
    if ((rc = run_cache(layers, E, layers * E, layers, 2, 2 * E + 2, 0, 20))) return 40 + rc;
    // sizing closed forms and capacities
    std::vector<int32_t> caps(layers);
    if (fate_cache_layer_capacities(layers, E, 40, 2, caps.data()) != FATE_OK) return 50;
    (void)fate_cache_total_from_budget(int64_t(8) << 30, int64_t(3) << 30, 4460544);
    (void)fate_n_max_from_times(7e-3, 5e-3, 1e-3, 6e-3);
    // co-activation statistics
    fate_eap* p = fate_eap_create(layers, E);
    if (!p) return 60;
    const int N = 9, k = 3;
    std::vector<int32_t> a(N * k), b(N * k), out(E);
    for (int it = 0; it < 20; ++it)
        for (int l = 0; l + 1 < layers; ++l) {
            for (int i = 0; i < N * k; ++i) { a[i] = (int)(rnd() % E); b[i] = (int)(rnd() % E); }
            if (fate_eap_update(p, l, a.data(), b.data(), N, k) != FATE_OK) return 61;
        }
    for (int l = 0; l < layers; ++l)
        if (fate_eap_predict(p, l, a.data(), N, k, 4, out.data()) != FATE_OK) return 62;
    fate_eap_destroy(p);
    printf("cache sanitizer driver: ok\n");
    return 0;
}
