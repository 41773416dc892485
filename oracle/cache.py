"""CPU oracle for the expert-cache step: sizing formulas, per-layer ARC and
the per-layer residency / prefetch / eviction bookkeeping.

TEST INFRASTRUCTURE ONLY.  Pure Python, integer logic; shares no code with
the library's C++ cache.

Paper basis: memory-budget model and shallow-favoring allocation (section
4.4: cache_total formula; boundary L, sequential fill of the first L layers
when memory is short, otherwise cache_deep per deep layer); ARC with queues
T1, T2, B1, B2 per layer (section 4.4, last paragraph; the replacement rules
are the published ARC algorithm); residency check and transfer of predicted
experts, cache-list update from the true gate result and eviction (section
4.1 steps 3-4 and 7-8); transfers in descending popularity and the cap n on
transfers per layer (section 4.3, prefill and decoding stages); compute order
"already on the device first, then in load order" (figure "rearranging the
order of expert computations").

The paper gives prose only; the readings taken here (floor divisions, the
order of tie-breaks, integer ARC adaptation step, prefetches not counted as
ARC accesses, slots freed in one step reusable from the next) are listed in
the design notes of the repository.
"""


def cache_total_from_budget(memory_budget, others, expert_bytes):
    """cache_total = (memory_budget - others) / expert, floored, >= 0."""
    if expert_bytes <= 0:
        raise ValueError("expert_bytes")
    return max(0, (int(memory_budget) - int(others)) // int(expert_bytes))


def n_max_from_times(t_moe, t_attn, t_gate, t_expert):
    """n = T / t_expert with T = t_moe + t_attn + t_gate, floored."""
    T = t_moe + t_attn + t_gate
    return int(T // t_expert)


def layer_capacities(num_layers, E, cache_total, L):
    """Shallow-favoring split of cache_total expert slots over layers."""
    L = max(0, min(L, num_layers))
    caps = [0] * num_layers
    if cache_total <= L * E:
        rem = cache_total
        for l in range(L):
            caps[l] = min(E, rem)
            rem -= caps[l]
        return caps
    for l in range(L):
        caps[l] = E
    deep = num_layers - L
    if deep > 0:
        rem = cache_total - L * E
        base, extra = divmod(rem, deep)
        for i in range(deep):
            caps[L + i] = min(E, base + (1 if i < extra else 0))
    return caps


class ARC:
    """Adaptive Replacement Cache over expert ids, capacity c >= 1.
    Lists hold LRU at index 0 and MRU at the end."""

    def __init__(self, c, preload=()):
        assert c >= 1
        self.c = c
        self.p = 0
        self.T1 = list(preload)
        self.T2 = []
        self.B1 = []
        self.B2 = []
        assert len(self.T1) <= c

    def resident(self, x):
        return x in self.T1 or x in self.T2

    def _replace(self, x_in_b2):
        t1 = len(self.T1)
        from_t1 = t1 >= 1 and (t1 > self.p or (x_in_b2 and t1 == self.p))
        if from_t1 or not self.T2:
            v = self.T1.pop(0)
            self.B1.append(v)
        else:
            v = self.T2.pop(0)
            self.B2.append(v)
        return v

    def access(self, x):
        """Reference to x.  Returns (was_resident, evicted_or_None)."""
        c = self.c
        if x in self.T1:
            self.T1.remove(x)
            self.T2.append(x)
            return True, None
        if x in self.T2:
            self.T2.remove(x)
            self.T2.append(x)
            return True, None
        if x in self.B1:
            delta = max(1, len(self.B2) // len(self.B1))
            self.p = min(c, self.p + delta)
            ev = self._replace(False)
            self.B1.remove(x)
            self.T2.append(x)
            return False, ev
        if x in self.B2:
            delta = max(1, len(self.B1) // len(self.B2))
            self.p = max(0, self.p - delta)
            ev = self._replace(True)
            self.B2.remove(x)
            self.T2.append(x)
            return False, ev
        ev = None
        l1 = len(self.T1) + len(self.B1)
        if l1 == c:
            if len(self.T1) < c:
                self.B1.pop(0)
                ev = self._replace(False)
            else:
                ev = self.T1.pop(0)
        else:
            total = l1 + len(self.T2) + len(self.B2)
            if total >= c:
                if total == 2 * c:
                    self.B2.pop(0)
                ev = self._replace(False)
        self.T1.append(x)
        return False, ev


class StepResult:
    def __init__(self):
        self.hit_cache = []      # experts found in the layer's cache
        self.hit_prefetch = []   # experts found staged by an earlier prefetch
        self.miss = []           # experts loaded on demand, in load order
        self.compute_order = []  # cached, then prefetched, then misses in load order
        self.loads = []          # (layer, expert, slot, is_demand) in issue order
        self.load_bits = []      # code width of each load (same order): the cache's width, or the low one
        self.slot_of = {}        # expert -> slot for every activated expert
        self.wasted = []         # staged-but-unused experts evicted at step start
        self.evicted = []        # experts evicted by ARC in this step
        self.prefetch_dropped = 0
        self.pair_hits = 0
        self.pair_misses = 0


class CacheOracle:
    """Reference simulator of the per-layer cache step."""

    def __init__(self, num_layers, E, cache_total, L_shallow, n_max, staging_slots, low_percent=0, bits=4,
                 low_bits=2):
        """low_percent: popularity-aware hybrid width of section 4.5 - of the experts predicted for
        the next layer, ranked by predicted popularity, the least popular low_percent % (floored) are
        transferred as low_bits copies when they need a transfer at all.  Such a copy serves the
        layer's computation and is then dropped: the cache holds `bits` copies only."""
        self.num_layers = num_layers
        self.E = E
        self.n_max = n_max
        self.low_percent, self.bits, self.low_bits = low_percent, bits, low_bits
        self.staged_low = [set() for _ in range(num_layers)]
        self.caps = layer_capacities(num_layers, E, cache_total, L_shallow)
        self.total_slots = sum(self.caps) + staging_slots
        self.full = [c >= E for c in self.caps]
        self.arc = [None] * num_layers
        self.slot = [dict() for _ in range(num_layers)]   # layer -> expert -> slot
        self.staged = [[] for _ in range(num_layers)]
        nxt = 0
        for l in range(num_layers):
            c = self.caps[l]
            n0 = E if self.full[l] else c
            for e in range(n0):
                self.slot[l][e] = nxt
                nxt += 1
            if not self.full[l] and c >= 1:
                self.arc[l] = ARC(c, preload=range(c))
        self.free = list(range(nxt, self.total_slots))   # ascending; lowest taken first
        self.pending = []

    # -- helpers -----------------------------------------------------------
    def resident(self, l, e):
        if self.full[l]:
            return True
        a = self.arc[l]
        return a is not None and a.resident(e)

    def _alloc(self):
        if not self.free:
            return None
        return self.free.pop(0)

    def _release(self, l, e):
        self.pending.append(self.slot[l].pop(e))

    # -- one step ------------------------------------------------------------
    def step(self, layer, actual_ids, actual_counts, pred_ids=(), pred_pop=()):
        r = StepResult()
        # slots freed during the previous step become reusable now
        self.free = sorted(self.free + self.pending)
        self.pending = []
        l = layer
        order = sorted(range(len(actual_ids)), key=lambda i: (-int(actual_counts[i]), i))
        A = [int(actual_ids[i]) for i in order]
        cnt = {int(actual_ids[i]): int(actual_counts[i]) for i in order}
        # (0) staged for this layer but not activated: wasted prefetches
        for e in list(self.staged[l]):
            if e not in cnt:
                self.staged[l].remove(e)
                self.staged_low[l].discard(e)
                self._release(l, e)
                r.wasted.append(e)
        # (i) residency check, demand loads
        for a in A:
            if self.resident(l, a):
                r.hit_cache.append(a)
                r.pair_hits += cnt[a]
            elif a in self.staged[l]:
                r.hit_prefetch.append(a)
                r.pair_hits += cnt[a]
            else:
                s = self._alloc()
                if s is None:
                    raise RuntimeError("no free slot for a demand load")
                self.slot[l][a] = s
                self.staged[l].append(a)
                r.miss.append(a)
                r.pair_misses += cnt[a]
                r.loads.append((l, a, s, True))
                r.load_bits.append(self.bits)
        # (ii) compute order
        r.compute_order = r.hit_cache + r.hit_prefetch + r.miss
        for a in A:
            r.slot_of[a] = self.slot[l][a]
        # (iii) cache-list update from the true routing, eviction.  The
        # accesses follow the compute order, so every expert that was a cache
        # hit is touched before any admission can evict it.
        if not self.full[l]:
            arc = self.arc[l]
            for a in r.compute_order:
                if arc is None or a in self.staged_low[l]:
                    # no cache in this layer, or a low-width copy: used once, then dropped
                    self.staged[l].remove(a)
                    self.staged_low[l].discard(a)
                    self._release(l, a)
                    r.evicted.append(a)
                    continue
                _, ev = arc.access(a)
                if a in self.staged[l]:
                    self.staged[l].remove(a)
                if ev is not None:
                    self._release(l, ev)
                    r.evicted.append(ev)
        # (iv) prefetch for the next layer from the prediction
        t = l + 1
        if t < self.num_layers and len(pred_ids) and self.n_max > 0:
            porder = sorted(range(len(pred_ids)), key=lambda i: (-int(pred_pop[i]), i))
            npos = sum(1 for i in porder if int(pred_pop[i]) > 0)
            nlow = npos * self.low_percent // 100
            rank = 0                      # position among the predicted experts with popularity > 0
            issued = 0
            for i in porder:
                if issued >= self.n_max:
                    break
                e = int(pred_ids[i])
                if int(pred_pop[i]) <= 0:
                    continue
                low = rank >= npos - nlow
                rank += 1
                if self.resident(t, e) or e in self.staged[t]:
                    continue
                s = self._alloc()
                if s is None:
                    r.prefetch_dropped += 1
                    continue
                self.slot[t][e] = s
                self.staged[t].append(e)
                if low:
                    self.staged_low[t].add(e)
                r.loads.append((t, e, s, False))
                r.load_bits.append(self.low_bits if low else self.bits)
                issued += 1
        return r


class EAPPredictor:
    """Activation-path predictor of the paper's EAP baseline (section 5.1): the experts of the
    next block are predicted from the token's expert choices in the previous block and
    statistics collected beforehand - here the co-activation counts
    freq[l][e][e'] = number of calibration tokens that chose e in block l and e' in block l+1.

    Reading (the paper gives one sentence): a token's score for a next-block expert is the sum of
    freq over the experts it chose; its prediction is the m experts with the highest positive
    scores, ties to the lower id; over a batch the predicted popularity of an expert is the
    number of tokens that predict it (the same aggregate the cross-layer prediction produces)."""

    def __init__(self, num_layers, E):
        self.num_layers, self.E = num_layers, E
        self.freq = [[[0] * E for _ in range(E)] for _ in range(max(0, num_layers - 1))]

    def update(self, layer, ids_l, ids_next):
        """ids_l, ids_next: [N][k] expert choices of the same tokens in blocks layer and layer+1."""
        f = self.freq[layer]
        for row, nxt in zip(ids_l, ids_next):
            for e in row:
                for e2 in nxt:
                    f[int(e)][int(e2)] += 1

    def predict(self, layer, ids_l, m):
        """Predicted popularity [E] of block layer+1 from the choices ids_l [N][k] in block layer."""
        pop = [0] * self.E
        if layer + 1 >= self.num_layers:
            return pop
        f = self.freq[layer]
        for row in ids_l:
            score = [0] * self.E
            for e in row:
                fe = f[int(e)]
                for e2 in range(self.E):
                    score[e2] += fe[e2]
            order = sorted(range(self.E), key=lambda e2: (-score[e2], e2))
            for e2 in order[:m]:
                if score[e2] > 0:
                    pop[e2] += 1
        return pop
