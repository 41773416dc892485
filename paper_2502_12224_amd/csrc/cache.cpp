// Expert cache policy: sizing closed forms, per-layer ARC, and the per-layer
// cache step (residency check, demand loads, compute order, cache-list update
// and eviction, prefetch for the next layer).  Host integer logic only; data
// movement goes through the copy callback, so this file needs no GPU.
//
// Paper section 4.4 (memory budget, boundary L, cache_deep, ARC per layer),
// section 4.1 steps 3-4 and 7-8, section 4.3 (popularity order, cap n).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <set>
#include <vector>

#include "../../include/fate.h"

namespace fate {
void set_error(const char* fmt, ...);
}

namespace {

enum Where : uint8_t { ABSENT = 0, IN_T1, IN_T2, IN_B1, IN_B2 };

// Adaptive Replacement Cache over expert ids 0..E-1; front of a list = LRU.
struct Arc {
    int c = 0, p = 0;
    std::vector<int> t1, t2, b1, b2;
    std::vector<uint8_t> where;

    void init(int cap, int E) {
        c = cap;
        p = 0;
        where.assign(E, ABSENT);
        for (int e = 0; e < cap && e < E; ++e) {
            t1.push_back(e);
            where[e] = IN_T1;
        }
    }
    bool resident(int x) const { return where[x] == IN_T1 || where[x] == IN_T2; }
    static void drop(std::vector<int>& l, int x) { l.erase(std::find(l.begin(), l.end(), x)); }
    int pop_lru(std::vector<int>& l) {
        int v = l.front();
        l.erase(l.begin());
        return v;
    }
    void push(std::vector<int>& l, int x, Where w) {
        l.push_back(x);
        where[x] = w;
    }
    // moves the LRU of T1 (or T2) to its ghost list and returns it
    int replace(bool x_in_b2) {
        const int n1 = (int)t1.size();
        const bool from_t1 = n1 >= 1 && (n1 > p || (x_in_b2 && n1 == p));
        if (from_t1 || t2.empty()) {
            int v = pop_lru(t1);
            push(b1, v, IN_B1);
            return v;
        }
        int v = pop_lru(t2);
        push(b2, v, IN_B2);
        return v;
    }
    // reference to x; returns the expert that lost its place, or -1
    int access(int x) {
        switch (where[x]) {
            case IN_T1: drop(t1, x); push(t2, x, IN_T2); return -1;
            case IN_T2: drop(t2, x); push(t2, x, IN_T2); return -1;
            case IN_B1: {
                int delta = std::max(1, (int)b2.size() / (int)b1.size());
                p = std::min(c, p + delta);
                int ev = replace(false);
                drop(b1, x);
                push(t2, x, IN_T2);
                return ev;
            }
            case IN_B2: {
                int delta = std::max(1, (int)b1.size() / (int)b2.size());
                p = std::max(0, p - delta);
                int ev = replace(true);
                drop(b2, x);
                push(t2, x, IN_T2);
                return ev;
            }
            default: break;
        }
        int ev = -1;
        const int l1 = (int)t1.size() + (int)b1.size();
        if (l1 == c) {
            if ((int)t1.size() < c) {
                where[pop_lru(b1)] = ABSENT;
                ev = replace(false);
            } else {
                ev = pop_lru(t1);
                where[ev] = ABSENT;
            }
        } else {
            const int total = l1 + (int)t2.size() + (int)b2.size();
            if (total >= c) {
                if (total == 2 * c) where[pop_lru(b2)] = ABSENT;
                ev = replace(false);
            }
        }
        push(t1, x, IN_T1);
        return ev;
    }
};

void capacities(int num_layers, int E, long long cache_total, int L, std::vector<int>& caps) {
    L = std::max(0, std::min(L, num_layers));
    caps.assign(num_layers, 0);
    if (cache_total <= (long long)L * E) {
        long long rem = std::max(0LL, cache_total);
        for (int l = 0; l < L; ++l) {
            caps[l] = (int)std::min<long long>(E, rem);
            rem -= caps[l];
        }
        return;
    }
    for (int l = 0; l < L; ++l) caps[l] = E;
    const int deep = num_layers - L;
    if (deep > 0) {
        const long long rem = cache_total - (long long)L * E;
        const long long base = rem / deep, extra = rem % deep;
        for (int i = 0; i < deep; ++i) caps[L + i] = (int)std::min<long long>(E, base + (i < extra ? 1 : 0));
    }
}

}  // namespace

struct fate_cache {
    int num_layers, E, n_max, total_slots;
    std::vector<int> caps;
    std::vector<uint8_t> full;
    std::vector<Arc> arc;                    // used when 0 < cap < E
    std::vector<std::vector<int>> slot;      // [layer][expert] -> slot or -1
    std::vector<std::vector<int>> staged;    // [layer] experts staged, in arrival order
    std::vector<std::vector<uint8_t>> staged_low;   // [layer][expert] 1 = the staged copy is the low-width one
    int bits = 4, low_bits = 2, low_percent = 0;
    std::set<int> free_slots;
    std::vector<int> pending;                // freed in the current step
    fate_copy_fn copy;
    void* user;

    bool resident(int l, int e) const { return full[l] || (caps[l] > 0 && arc[l].resident(e)); }
    bool is_staged(int l, int e) const {
        return std::find(staged[l].begin(), staged[l].end(), e) != staged[l].end();
    }
    void unstage(int l, int e) { staged[l].erase(std::find(staged[l].begin(), staged[l].end(), e)); }
    void release(int l, int e) {
        pending.push_back(slot[l][e]);
        slot[l][e] = -1;
    }
    int alloc() {
        if (free_slots.empty()) return -1;
        int s = *free_slots.begin();
        free_slots.erase(free_slots.begin());
        return s;
    }
};

extern "C" int64_t fate_cache_total_from_budget(int64_t memory_budget, int64_t others, int64_t expert_bytes) {
    if (expert_bytes <= 0) return -1;
    const int64_t room = memory_budget - others;
    return room <= 0 ? 0 : room / expert_bytes;
}

extern "C" int32_t fate_n_max_from_times(double t_moe, double t_attn, double t_gate, double t_expert) {
    if (!(t_expert > 0)) return -1;
    const double n = std::floor((t_moe + t_attn + t_gate) / t_expert);
    return n < 0 ? 0 : (n > 2147483647.0 ? 2147483647 : (int32_t)n);
}

extern "C" fate_status fate_cache_layer_capacities(int num_layers, int E, int cache_total, int L_shallow,
                                                   int32_t* caps) {
    if (num_layers < 1 || E < 1 || cache_total < 0 || L_shallow < 0 || caps == nullptr) {
        fate::set_error("fate_cache_layer_capacities: bad argument");
        return FATE_EINVAL;
    }
    std::vector<int> c;
    capacities(num_layers, E, cache_total, L_shallow, c);
    for (int l = 0; l < num_layers; ++l) caps[l] = c[l];
    return FATE_OK;
}

extern "C" fate_cache* fate_cache_create(int num_layers, int E, int cache_total, int L_shallow, int n_max,
                                         int staging_slots, fate_copy_fn copy, void* user) {
    if (num_layers < 1 || E < 1 || E > 256 || cache_total < 0 || L_shallow < 0 || n_max < 0 ||
        staging_slots < 0) {
        fate::set_error("fate_cache_create: bad argument");
        return nullptr;
    }
    fate_cache* c = new fate_cache();
    c->num_layers = num_layers;
    c->E = E;
    c->n_max = n_max;
    c->copy = copy;
    c->user = user;
    capacities(num_layers, E, cache_total, L_shallow, c->caps);
    c->full.resize(num_layers);
    c->arc.resize(num_layers);
    c->slot.assign(num_layers, std::vector<int>(E, -1));
    c->staged.resize(num_layers);
    c->staged_low.assign(num_layers, std::vector<uint8_t>(E, 0));
    int next = 0;
    for (int l = 0; l < num_layers; ++l) {
        c->full[l] = c->caps[l] >= E;
        const int n0 = c->full[l] ? E : c->caps[l];
        for (int e = 0; e < n0; ++e) c->slot[l][e] = next++;
        if (!c->full[l] && c->caps[l] >= 1) c->arc[l].init(c->caps[l], E);
    }
    c->total_slots = next + staging_slots;
    for (int s = next; s < c->total_slots; ++s) c->free_slots.insert(s);
    return c;
}

extern "C" void fate_cache_destroy(fate_cache* c) { delete c; }
extern "C" int32_t fate_cache_total_slots(const fate_cache* c) { return c ? c->total_slots : -1; }
extern "C" fate_status fate_cache_set_n_max(fate_cache* c, int n_max) {
    if (!c || n_max < 0) {
        fate::set_error("fate_cache_set_n_max: cache %p, n_max %d", (void*)c, n_max);
        return FATE_EINVAL;
    }
    c->n_max = n_max;
    return FATE_OK;
}
extern "C" fate_status fate_cache_set_low_precision(fate_cache* c, int percent, int bits, int low_bits) {
    if (!c || percent < 0 || percent > 100 || bits < 1 || low_bits < 1) {
        fate::set_error("fate_cache_set_low_precision: cache %p, percent %d, bits %d / %d", (void*)c, percent, bits,
                        low_bits);
        return FATE_EINVAL;
    }
    c->low_percent = percent;
    c->bits = bits;
    c->low_bits = low_bits;
    return FATE_OK;
}
extern "C" int32_t fate_cache_slot_of(const fate_cache* c, int layer, int expert) {
    if (!c || layer < 0 || layer >= c->num_layers || expert < 0 || expert >= c->E) return -1;
    return c->slot[layer][expert];
}
extern "C" int32_t fate_cache_resident(const fate_cache* c, int layer, int expert) {
    if (!c || layer < 0 || layer >= c->num_layers || expert < 0 || expert >= c->E) return 0;
    if (c->resident(layer, expert)) return 2;
    return c->is_staged(layer, expert) ? 1 : 0;
}

extern "C" fate_status fate_expert_cache_step(fate_cache* c, int layer, const int32_t* actual_ids,
                                              const int32_t* actual_counts, int n_actual,
                                              const int32_t* pred_ids, const int32_t* pred_pop, int n_pred,
                                              int32_t* compute_order, int32_t* slots, fate_cache_load* loads,
                                              int max_loads, fate_cache_stats* stats) {
    if (!c) { fate::set_error("cache is NULL"); return FATE_EINVAL; }
    if (layer < 0 || layer >= c->num_layers) { fate::set_error("layer %d out of range", layer); return FATE_EINVAL; }
    if (n_actual < 0 || n_pred < 0 || (n_actual && (!actual_ids || !actual_counts || !compute_order || !slots)) ||
        (n_pred && (!pred_ids || !pred_pop)) || !stats || (max_loads > 0 && !loads) || max_loads < 0) {
        fate::set_error("fate_expert_cache_step: bad argument");
        return FATE_EINVAL;
    }
    const int E = c->E, l = layer;
    std::vector<int> cnt(E, 0);
    for (int i = 0; i < n_actual; ++i) {
        const int e = actual_ids[i];
        if (e < 0 || e >= E || actual_counts[i] <= 0 || cnt[e] != 0) {
            fate::set_error("actual_ids must be unique ids in [0,E) with positive counts");
            return FATE_EINVAL;
        }
        cnt[e] = actual_counts[i];
    }
    for (int i = 0; i < n_pred; ++i)
        if (pred_ids[i] < 0 || pred_ids[i] >= E) {
            fate::set_error("pred_ids out of range");
            return FATE_EINVAL;
        }
    fate_cache_stats st{};
    auto record = [&](int ly, int e, int s, int demand, int bits) {
        if (st.n_loads < max_loads) loads[st.n_loads] = fate_cache_load{ly, e, s, demand, bits};
        ++st.n_loads;
    };
    // slots released during the previous step are reusable from here on
    for (int s : c->pending) c->free_slots.insert(s);
    c->pending.clear();

    std::vector<int> order(n_actual);
    for (int i = 0; i < n_actual; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return actual_counts[a] > actual_counts[b]; });

    // prefetched for this layer but not activated
    {
        std::vector<int> keep;
        for (int e : c->staged[l]) {
            if (cnt[e] == 0) {
                c->release(l, e);
                c->staged_low[l][e] = 0;
                ++st.n_wasted;
            } else {
                keep.push_back(e);
            }
        }
        c->staged[l].swap(keep);
    }
    // residency check; demand loads
    std::vector<int> hit_cache, hit_pref, miss;
    for (int i : order) {
        const int e = actual_ids[i];
        if (c->resident(l, e)) {
            hit_cache.push_back(e);
            st.pair_hits += cnt[e];
        } else if (c->is_staged(l, e)) {
            hit_pref.push_back(e);
            st.pair_hits += cnt[e];
        } else {
            const int s = c->alloc();
            if (s < 0) {
                *stats = st;
                fate::set_error("layer %d: no free slot for the demand load of expert %d", l, e);
                return FATE_ECAPACITY;
            }
            if (c->copy && c->copy(c->user, l, e, s, 1, c->bits) != 0) {
                c->free_slots.insert(s);
                *stats = st;
                fate::set_error("layer %d: copy of expert %d into slot %d failed", l, e, s);
                return FATE_EHIP;
            }
            c->slot[l][e] = s;
            c->staged[l].push_back(e);
            miss.push_back(e);
            st.pair_misses += cnt[e];
            record(l, e, s, 1, c->bits);
        }
    }
    st.n_hit_cache = (int)hit_cache.size();
    st.n_hit_prefetch = (int)hit_pref.size();
    st.n_miss = (int)miss.size();
    // compute order: cached, prefetched, then demand-loaded in load order
    int w = 0;
    for (const std::vector<int>* v : {&hit_cache, &hit_pref, &miss})
        for (int e : *v) {
            compute_order[w] = e;
            slots[w] = c->slot[l][e];
            ++w;
        }
    // cache-list update from the true routing (in compute order), eviction
    if (!c->full[l]) {
        for (int i = 0; i < n_actual; ++i) {
            const int e = compute_order[i];
            if (c->caps[l] == 0 || c->staged_low[l][e]) {
                // no cache in this layer, or a low-width copy: used once, then dropped
                c->unstage(l, e);
                c->staged_low[l][e] = 0;
                c->release(l, e);
                ++st.n_evicted;
                continue;
            }
            const int ev = c->arc[l].access(e);
            if (c->is_staged(l, e)) c->unstage(l, e);
            if (ev >= 0) {
                c->release(l, ev);
                ++st.n_evicted;
            }
        }
    }
    // prefetch for the next layer, most popular first, at most n_max
    const int t = l + 1;
    if (t < c->num_layers && n_pred > 0 && c->n_max > 0) {
        std::vector<int> po(n_pred);
        for (int i = 0; i < n_pred; ++i) po[i] = i;
        std::stable_sort(po.begin(), po.end(), [&](int a, int b) { return pred_pop[a] > pred_pop[b]; });
        // popularity-aware hybrid width (section 4.5): the least popular low_percent % of the predicted
        // experts travel as low-width copies when they need a transfer
        int npos = 0;
        for (int i : po) npos += pred_pop[i] > 0;
        const int nlow = (int)((long long)npos * c->low_percent / 100);
        int rank = 0, issued = 0;
        for (int i : po) {
            if (issued >= c->n_max) break;
            const int e = pred_ids[i];
            if (pred_pop[i] <= 0) continue;
            const bool low = rank >= npos - nlow;
            ++rank;
            if (c->resident(t, e) || c->is_staged(t, e)) continue;
            const int s = c->alloc();
            if (s < 0) {
                ++st.n_prefetch_dropped;
                continue;
            }
            const int bits = low ? c->low_bits : c->bits;
            if (c->copy && c->copy(c->user, t, e, s, 0, bits) != 0) {
                c->free_slots.insert(s);
                *stats = st;
                fate::set_error("layer %d: prefetch copy of expert %d into slot %d failed", t, e, s);
                return FATE_EHIP;
            }
            c->slot[t][e] = s;
            c->staged[t].push_back(e);
            c->staged_low[t][e] = low ? 1 : 0;
            record(t, e, s, 0, bits);
            ++issued;
        }
        st.n_prefetch_issued = issued;
    }
    *stats = st;
    return FATE_OK;
}

// ---- dense-count front ends -------------------------------------------------
// The device produces per-expert pair counts [E] (fate_permute) and predicted
// popularity [E] (fate_cross_layer_predict); these wrappers take those arrays
// as they are, in id order, and build the unique lists themselves.

extern "C" fate_status fate_expert_cache_step_dense(fate_cache* c, int layer, const int32_t* counts,
                                                    const int32_t* pred_pop, int32_t* compute_order,
                                                    int32_t* slots, int32_t* n_actual_out,
                                                    fate_cache_load* loads, int max_loads,
                                                    fate_cache_stats* stats) {
    if (!c || !counts || !compute_order || !slots || !stats) {
        fate::set_error("fate_expert_cache_step_dense: bad argument");
        return FATE_EINVAL;
    }
    const int E = c->E;
    int32_t ids[256], cnt[256], pids[256], ppop[256];
    int n = 0, np = 0;
    for (int e = 0; e < E; ++e)
        if (counts[e] > 0) { ids[n] = e; cnt[n] = counts[e]; ++n; }
    if (pred_pop)
        for (int e = 0; e < E; ++e)
            if (pred_pop[e] > 0) { pids[np] = e; ppop[np] = pred_pop[e]; ++np; }
    if (n_actual_out) *n_actual_out = n;
    return fate_expert_cache_step(c, layer, ids, cnt, n, pids, ppop, np, compute_order, slots, loads, max_loads,
                                  stats);
}

extern "C" fate_status fate_expert_cache_step_layers(fate_cache* c, int layer_begin, int layer_end,
                                                     const int32_t* counts, const int32_t* pred_pop,
                                                     fate_cache_stats* stats_sum) {
    if (!c || !counts || !stats_sum || layer_begin < 0 || layer_end > c->num_layers || layer_begin > layer_end) {
        fate::set_error("fate_expert_cache_step_layers: bad argument");
        return FATE_EINVAL;
    }
    for (int l = layer_begin; l < layer_end; ++l)
        if (!c->full[l]) {
            fate::set_error("layer %d is not fully cached: step it on its own", l);
            return FATE_ENOTRESIDENT;
        }
    fate_cache_stats sum{};
    int32_t order[256], slots[256];
    for (int l = layer_begin; l < layer_end; ++l) {
        fate_cache_stats st{};
        const size_t o = (size_t)(l - layer_begin) * c->E;
        fate_status s = fate_expert_cache_step_dense(c, l, counts + o, pred_pop ? pred_pop + o : nullptr, order,
                                                     slots, nullptr, nullptr, 0, &st);
        if (s != FATE_OK) return s;
        sum.n_hit_cache += st.n_hit_cache; sum.n_hit_prefetch += st.n_hit_prefetch; sum.n_miss += st.n_miss;
        sum.pair_hits += st.pair_hits; sum.pair_misses += st.pair_misses;
        sum.n_prefetch_issued += st.n_prefetch_issued; sum.n_prefetch_dropped += st.n_prefetch_dropped;
        sum.n_wasted += st.n_wasted; sum.n_evicted += st.n_evicted; sum.n_loads += st.n_loads;
    }
    *stats_sum = sum;
    return FATE_OK;
}

// ---- activation-path predictor (the EAP baseline of section 5.1) ------------------------------
// Co-activation counts freq[l][e][e'] of calibration tokens between consecutive blocks; a token's
// prediction for block l+1 is the m experts with the highest positive summed counts over the
// experts it chose in block l (ties to the lower id); the predicted popularity of an expert is
// the number of tokens that predict it.  Host integer logic, a comparison mode for the cache step.
struct fate_eap {
    int num_layers, E;
    std::vector<int64_t> freq;      // [num_layers - 1][E][E]
};

extern "C" fate_eap* fate_eap_create(int num_layers, int E) {
    if (num_layers < 1 || E < 1 || E > 256) {
        fate::set_error("fate_eap_create: bad argument");
        return nullptr;
    }
    fate_eap* p = new fate_eap();
    p->num_layers = num_layers;
    p->E = E;
    p->freq.assign((size_t)std::max(0, num_layers - 1) * E * E, 0);
    return p;
}

extern "C" void fate_eap_destroy(fate_eap* p) { delete p; }

static bool eap_ids_ok(const fate_eap* p, const int32_t* ids, int n) {
    for (int i = 0; i < n; ++i)
        if (ids[i] < 0 || ids[i] >= p->E) return false;
    return true;
}

extern "C" fate_status fate_eap_update(fate_eap* p, int layer, const int32_t* ids_l, const int32_t* ids_next, int N,
                                       int k) {
    if (!p || layer < 0 || layer + 1 >= p->num_layers || N < 0 || k < 1 || (N && (!ids_l || !ids_next)) ||
        !eap_ids_ok(p, ids_l, N * k) || !eap_ids_ok(p, ids_next, N * k)) {
        fate::set_error("fate_eap_update: bad argument");
        return FATE_EINVAL;
    }
    int64_t* f = p->freq.data() + (size_t)layer * p->E * p->E;
    for (int t = 0; t < N; ++t)
        for (int i = 0; i < k; ++i)
            for (int j = 0; j < k; ++j) ++f[(size_t)ids_l[t * k + i] * p->E + ids_next[t * k + j]];
    return FATE_OK;
}

extern "C" fate_status fate_eap_predict(const fate_eap* p, int layer, const int32_t* ids_l, int N, int k, int m,
                                        int32_t* pred_pop) {
    if (!p || layer < 0 || layer >= p->num_layers || N < 0 || k < 1 || m < 1 || !pred_pop || (N && !ids_l) ||
        !eap_ids_ok(p, ids_l, N * k)) {
        fate::set_error("fate_eap_predict: bad argument");
        return FATE_EINVAL;
    }
    const int E = p->E;
    for (int e = 0; e < E; ++e) pred_pop[e] = 0;
    if (layer + 1 >= p->num_layers) return FATE_OK;
    const int64_t* f = p->freq.data() + (size_t)layer * E * E;
    std::vector<int64_t> score(E);
    std::vector<int> order(E);
    for (int t = 0; t < N; ++t) {
        std::fill(score.begin(), score.end(), 0);
        for (int i = 0; i < k; ++i) {
            const int64_t* fe = f + (size_t)ids_l[t * k + i] * E;
            for (int e = 0; e < E; ++e) score[e] += fe[e];
        }
        for (int e = 0; e < E; ++e) order[e] = e;
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return score[a] > score[b]; });
        for (int i = 0; i < m && i < E; ++i)
            if (score[order[i]] > 0) ++pred_pop[order[i]];
    }
    return FATE_OK;
}
