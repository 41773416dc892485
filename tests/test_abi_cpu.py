"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, rejects bad arguments before touching a GPU, and its C++
cache policy reproduces the Python oracle on random traces."""
import ctypes as C
import os
import random
import re

import pytest

from oracle import cache as OC
import paper_2502_12224_amd.binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            txt = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, f)).read(), flags=re.S)
            names |= set(re.findall(r"\b(fate_[a-z0-9_]+)\s*\(", txt))
    return sorted(names - {"fate_copy_fn"})


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = _declared_symbols()
    assert len(names) >= 20 and set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(L, n), n
    assert b"gfx950" in L.fate_version()


def test_argument_validation_without_gpu():
    L = B.lib()
    z = C.c_void_p(0)
    p16 = C.c_void_p(0x1000)      # never dereferenced: validation fails first
    odd = C.c_void_p(0x1004)
    # routing
    assert L.fate_gate_route(z, p16, p16, z, 4, 2048, 0, 1, 0, p16, p16, z) == 2          # E = 0
    assert L.fate_gate_route(z, p16, p16, z, 4, 2048, 300, 1, 0, p16, p16, z) == 2        # E > 256
    assert L.fate_gate_route(z, p16, p16, z, 4, 100, 8, 2, 0, p16, p16, z) == 2           # H % 64
    assert L.fate_gate_route(z, p16, p16, z, 4, 256, 8, 9, 0, p16, p16, z) == 1           # k > E
    assert L.fate_gate_route(z, z, p16, z, 4, 256, 8, 2, 0, p16, p16, z) == 1             # NULL x
    assert L.fate_gate_route(z, odd, p16, z, 4, 256, 8, 2, 0, p16, p16, z) == 3           # misaligned
    assert b"aligned" in L.fate_last_error()
    assert L.fate_gate_route(z, z, z, z, 0, 256, 8, 2, 0, z, z, z) == 0                   # N = 0: nothing to do
    assert L.fate_cross_layer_predict(z, p16, p16, z, 4, 256, 8, 4, 2, p16, p16, p16) == 1   # m < k
    assert L.fate_cross_layer_predict(z, p16, p16, z, 4, 256, 8, 2, 9, p16, p16, p16) == 1   # m > E
    assert L.fate_permute(z, p16, 4, 0, 8, p16, p16, p16, p16, p16) == 1                  # k = 0
    assert L.fate_permute(z, p16, 4, 2, 8, z, p16, p16, p16, p16) == 1                    # NULL counts
    # fused routing: workspace too small, N between the decode and the prefill range, prefill N with an unsuitable H
    nb = C.c_size_t(0)
    assert L.fate_route_fused_workspace(4, 60, C.byref(nb)) == 0 and nb.value == 256 + 2 * 4 * 60 * 4
    args = [z, p16, p16, z, p16, z, 4, 2048, 60, 4, 15, 0] + [p16] * 10
    assert L.fate_route_fused(*args, p16, C.c_size_t(16)) == 4
    args[6] = 32
    assert L.fate_route_fused(*args, p16, C.c_size_t(1 << 20)) == 2
    args[6], args[7] = 64, 1536
    assert L.fate_route_fused(*args, p16, C.c_size_t(1 << 20)) == 2
    # packing
    assert L.fate_pack_weight(z, p16, 32, 64, 3, C.c_void_p(0x2000)) == 1
    assert L.fate_pack_weight(z, p16, 40, 64, 4, C.c_void_p(0x2000)) == 2
    assert L.fate_pack_weight(z, p16, 32, 64, 4, p16) == 1                                # in place
    # FFN descriptor
    d = B.make_ffn_desc(4, 2048, 60, 4, 1408, 4, 128, 1, 5632, 4, 128)
    nb = C.c_size_t(0)
    assert L.fate_moe_ffn_q_workspace(C.byref(d), C.byref(nb)) == 0
    assert nb.value >= 4 * 4 * 1408 * 2 + 4 * 5632 * 2
    bad = B.make_ffn_desc(4, 2048, 60, 4, 1408, 5, 128)
    assert L.fate_moe_ffn_q_workspace(C.byref(bad), C.byref(nb)) == 1
    bad = B.make_ffn_desc(4, 2048, 60, 4, 1400, 4, 128)
    assert L.fate_moe_ffn_q_workspace(C.byref(bad), C.byref(nb)) == 2
    assert L.fate_moe_ffn_q(z, C.byref(d), p16, p16, p16, p16, p16, p16, p16, p16, p16, z, p16, p16, C.c_size_t(8)) == 4
    d0 = B.make_ffn_desc(0, 2048, 60, 4, 1408, 4, 128)
    assert L.fate_moe_ffn_q(z, C.byref(d0), z, z, z, z, z, z, z, z, z, z, z, z, C.c_size_t(0)) == 0


def test_closed_forms_match_oracle():
    L = B.lib()
    rnd = random.Random(3)
    for _ in range(200):
        b, o, e = rnd.randint(0, 1 << 36), rnd.randint(0, 1 << 35), rnd.randint(1, 1 << 27)
        assert L.fate_cache_total_from_budget(b, o, e) == OC.cache_total_from_budget(b, o, e)
        nl, E = rnd.randint(1, 40), rnd.randint(1, 70)
        Ls, total = rnd.randint(0, nl + 2), rnd.randint(0, nl * E + 10)
        caps = (C.c_int32 * nl)()
        assert L.fate_cache_layer_capacities(nl, E, total, Ls, caps) == 0
        assert list(caps) == OC.layer_capacities(nl, E, total, Ls)
    assert L.fate_n_max_from_times(13.0, 0.0, 0.0, 6.0) == 2
    assert L.fate_n_max_from_times(0.1, 0.1, 0.1, 1.0) == 0


class _Cache:
    """The C++ cache driven through the C ABI with a recording copy callback."""

    def __init__(self, nl, E, total, Ls, n_max, staging, fail_at=None):
        self.copies = []
        self.copy_bits = []
        self.fail_at = fail_at

        def cb(user, layer, expert, slot, demand, bits):
            if self.fail_at is not None and len(self.copies) == self.fail_at:
                return 1
            self.copies.append((layer, expert, slot, bool(demand)))
            self.copy_bits.append(bits)
            return 0
        self._cb = B.COPY_FN(cb)
        self.h = B.lib().fate_cache_create(nl, E, total, Ls, n_max, staging, self._cb, None)
        assert self.h

    def step(self, layer, ids, counts, pids=(), ppop=()):
        n, npred = len(ids), len(pids)
        a = (C.c_int32 * max(n, 1))(*ids)
        c = (C.c_int32 * max(n, 1))(*counts)
        pi = (C.c_int32 * max(npred, 1))(*pids)
        pp = (C.c_int32 * max(npred, 1))(*ppop)
        order = (C.c_int32 * max(n, 1))()
        slots = (C.c_int32 * max(n, 1))()
        loads = (B.fate_cache_load * 512)()
        st = B.fate_cache_stats()
        rc = B.lib().fate_expert_cache_step(self.h, layer, a, c, n, pi, pp, npred, order, slots, loads, 512,
                                            C.byref(st))
        ld = [(loads[i].layer, loads[i].expert, loads[i].slot, bool(loads[i].demand)) for i in range(min(st.n_loads, 512))]
        self.last_bits = [loads[i].bits for i in range(min(st.n_loads, 512))]
        return rc, list(order)[:n], list(slots)[:n], ld, st

    def close(self):
        B.lib().fate_cache_destroy(self.h)


@pytest.mark.parametrize("seed", range(6))
def test_cpp_cache_matches_oracle_on_random_traces(seed):
    rnd = random.Random(seed)
    nl, E = rnd.randint(2, 6), rnd.choice([8, 16, 60])
    k = rnd.randint(1, 4)
    total = rnd.randint(0, nl * E)
    Ls = rnd.randint(0, 3)
    n_max = rnd.randint(0, 5)
    staging = 3 * E
    ref = OC.CacheOracle(nl, E, total, Ls, n_max, staging)
    cc = _Cache(nl, E, total, Ls, n_max, staging)
    assert B.lib().fate_cache_total_slots(cc.h) == ref.total_slots
    hot = [rnd.sample(range(E), min(E, 6)) for _ in range(nl)]
    for it in range(120):
        for l in range(nl):
            ntok = rnd.choice([1, 1, 4, 30])
            cnt = {}
            for _ in range(ntok * k):
                e = rnd.choice(hot[l]) if rnd.random() < 0.6 else rnd.randrange(E)
                cnt[e] = cnt.get(e, 0) + 1
            ids = sorted(cnt)
            counts = [cnt[e] for e in ids]
            pc = {}
            for _ in range(ntok * (k + 2)):
                e = rnd.choice(hot[(l + 1) % nl]) if rnd.random() < 0.7 else rnd.randrange(E)
                pc[e] = pc.get(e, 0) + 1
            pids = sorted(pc)
            ppop = [pc[e] for e in pids]
            r = ref.step(l, ids, counts, pids, ppop)
            rc, order, slots, loads, st = cc.step(l, ids, counts, pids, ppop)
            assert rc == 0
            assert order == r.compute_order
            assert slots == [r.slot_of[e] for e in r.compute_order]
            assert loads == r.loads
            assert (st.n_hit_cache, st.n_hit_prefetch, st.n_miss) == (len(r.hit_cache), len(r.hit_prefetch), len(r.miss))
            assert (st.pair_hits, st.pair_misses) == (r.pair_hits, r.pair_misses)
            assert st.n_wasted == len(r.wasted) and st.n_evicted == len(r.evicted)
            assert st.n_prefetch_dropped == r.prefetch_dropped
            for e in range(E):
                want = 2 if ref.resident(l, e) else (1 if e in ref.staged[l] else 0)
                assert B.lib().fate_cache_resident(cc.h, l, e) == want
                assert B.lib().fate_cache_slot_of(cc.h, l, e) == ref.slot[l].get(e, -1)
    assert cc.copies == [ld for ld in cc.copies]       # callback saw every load exactly once
    cc.close()


def test_cache_set_n_max_changes_the_prefetch_cap():
    # section 4.3: the cap n is re-derived per phase; the C++ cache follows the oracle after a change
    nl, E = 3, 16
    ref = OC.CacheOracle(nl, E, 6, 0, 0, 2 * E)
    cc = _Cache(nl, E, 6, 0, 0, 2 * E)
    assert B.lib().fate_cache_set_n_max(cc.h, -1) == 1
    for n_max in (0, 3, 16, 1):
        ref.n_max = n_max
        assert B.lib().fate_cache_set_n_max(cc.h, n_max) == 0
        for l in range(nl):
            ids, counts = [1, 5, 9], [2, 1, 1]
            pids, ppop = list(range(4, 12)), [8, 7, 6, 5, 4, 3, 2, 1]
            r = ref.step(l, ids, counts, pids, ppop)
            rc, order, slots, loads, st = cc.step(l, ids, counts, pids, ppop)
            assert rc == 0 and loads == r.loads and order == r.compute_order
            if l + 1 < nl:
                assert st.n_prefetch_issued <= n_max
    cc.close()


def test_cache_error_paths():
    # a failing copy is reported and the expert is not marked resident
    cc = _Cache(2, 8, 0, 0, 2, 8, fail_at=1)
    rc, *_ = cc.step(0, [1, 2], [1, 1])
    assert rc == 6 and b"copy" in B.lib().fate_last_error()
    assert B.lib().fate_cache_resident(cc.h, 0, 1) == 1 and B.lib().fate_cache_resident(cc.h, 0, 2) == 0
    cc.close()
    # no staging room for a demand load
    cc = _Cache(1, 8, 0, 0, 0, 1)
    rc, *_ = cc.step(0, [1, 2], [1, 1])
    assert rc == 7
    cc.close()
    # bad arguments
    cc = _Cache(2, 8, 4, 1, 1, 8)
    assert cc.step(5, [1], [1])[0] == 1
    assert cc.step(0, [1, 1], [1, 1])[0] == 1
    assert cc.step(0, [9], [1])[0] == 1
    assert cc.step(0, [1], [0])[0] == 1
    cc.close()
    assert not B.lib().fate_cache_create(0, 8, 4, 1, 1, 8, B.COPY_FN(0), None)


def test_bench_refuses_more_than_one_gpu():
    """The bench line is a one-GPU figure: asking for more ends with a message, before any GPU work."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0
    assert "one GPU" in p.stderr + p.stdout
    assert not any(l.startswith("{") for l in p.stdout.splitlines())


def test_eap_predictor_follows_the_oracle():
    """The C++ activation-path predictor against the Python one on random calibration data."""
    L = B.lib()
    nl, E, k, m = 4, 16, 3, 5
    rnd = random.Random(5)
    ref = OC.EAPPredictor(nl, E)
    h = L.fate_eap_create(nl, E)
    assert h
    arr = lambda rows: (C.c_int32 * (len(rows) * k))(*[e for r in rows for e in r])
    pick = lambda n: [rnd.sample(range(E), k) for _ in range(n)]
    for _ in range(20):
        for l in range(nl - 1):
            a, b = pick(7), pick(7)
            ref.update(l, a, b)
            assert L.fate_eap_update(h, l, arr(a), arr(b), 7, k) == 0
    out = (C.c_int32 * E)()
    for l in range(nl):
        q = pick(9)
        assert L.fate_eap_predict(h, l, arr(q), 9, k, m, out) == 0
        assert list(out) == ref.predict(l, q, m), l
    assert L.fate_eap_update(h, nl - 1, arr(pick(1)), arr(pick(1)), 1, k) == 1       # no block after the last
    assert L.fate_eap_predict(h, 0, arr([[0, 1, E]]), 1, k, m, out) == 1             # id out of range
    L.fate_eap_destroy(h)


def test_hybrid_width_of_the_prefetch_list_follows_the_oracle():
    """Popularity-aware hybrid width (section 4.5): the C++ cache against the oracle on random traces with
    the least popular quarter of the predicted experts moved as 2-bit copies, then with the rule off."""
    nl, E = 4, 16
    rnd = random.Random(17)
    for percent in (25, 50, 0):
        ref = OC.CacheOracle(nl, E, 14, 1, 6, 2 * E, low_percent=percent)
        cc = _Cache(nl, E, 14, 1, 6, 2 * E)
        assert B.lib().fate_cache_set_low_precision(cc.h, percent, 4, 2) == 0
        seen_low = 0
        for step in range(40):
            for l in range(nl):
                ids = sorted(rnd.sample(range(E), rnd.randint(1, 5)))
                counts = [rnd.randint(1, 9) for _ in ids]
                pids = sorted(rnd.sample(range(E), rnd.randint(0, 10)))
                ppop = [rnd.randint(0, 6) for _ in pids]
                r = ref.step(l, ids, counts, pids, ppop)
                rc, order, slots, loads, st = cc.step(l, ids, counts, pids, ppop)
                assert rc == 0 and order == r.compute_order and loads == r.loads
                assert cc.last_bits == r.load_bits
                assert st.n_evicted == len(r.evicted) and st.n_wasted == len(r.wasted)
                seen_low += sum(1 for b in r.load_bits if b == 2)
                for e in range(E):
                    want = 2 if ref.resident(l, e) else (1 if e in ref.staged[l] else 0)
                    assert B.lib().fate_cache_resident(cc.h, l, e) == want
        assert (seen_low > 0) == (percent > 0)
        assert cc.copy_bits.count(2) == seen_low
        cc.close()
    assert B.lib().fate_cache_set_low_precision(None, 25, 4, 2) == 1


def test_cache_policy_under_address_and_ub_sanitizers(tmp_path):
    """cache.cpp (host-only policy code) built with -fsanitize=address,undefined together with a driver that runs
    random traces through every mode of the cache step and the co-activation predictor: any report aborts the run."""
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    exe = str(tmp_path / "cache_san")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", os.path.join(root, "tests", "native", "cache_sanitizer_driver.cpp"),
           os.path.join(root, "paper_2502_12224_amd", "csrc", "cache.cpp"), "-o", exe]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "cache sanitizer driver: ok" in r.stdout
