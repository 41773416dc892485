"""Expert cache on the device: experts in a pinned host pool, copies on a side
stream through the built-in HIP engine.  Results must equal the all-resident
path, and the cache decisions must equal the Python cache oracle's."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import cache as OC
from paper_2502_12224_amd.stack import LayerBuffers, MoEStack, OffloadedStack, layer_forward
from workloads import SHAPES, chain_next_hidden, gen_hidden, unit_rmsnorm_bf16
from helpers import DEV

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,cache_total,n_max,L_shallow", [(1, 10, 2, 1), (3, 6, 1, 0), (2, 0, 0, 0), (2, 40, 3, 2)])
def test_offloaded_stack_matches_resident_and_oracle(N, cache_total, n_max, L_shallow):
    cfg = dataclasses.replace(SHAPES["tiny"], name="tiny4", layers=4)
    L, E = cfg.layers, cfg.E
    staging = 2 * E + n_max
    ref = MoEStack(cfg, DEV)
    off = OffloadedStack(cfg, cache_total, n_max, staging, DEV, L_shallow=L_shallow)
    off.keep_trace = True
    sim = OC.CacheOracle(L, E, cache_total, L_shallow, n_max, staging)
    assert off.caps == sim.caps and off.total_slots == sim.total_slots
    b_ref, b_off = LayerBuffers(cfg, N, DEV), LayerBuffers(cfg, N, DEV)
    hits = misses = 0
    for step in range(8):
        h = gen_hidden(cfg, N, step=step, device=DEV).float()
        for l in range(L):
            x = unit_rmsnorm_bf16(h)
            y_ref = layer_forward(cfg, ref.layers[l], ref.layers[l + 1] if l + 1 < L else None, x, b_ref).clone()
            ntr = len(off.trace)
            y_off = off.layer(l, x, b_off)
            torch.cuda.synchronize()
            assert torch.equal(b_ref.ids, b_off.ids) and torch.equal(b_ref.perm, b_off.perm)
            assert int(b_off.ffn_ws[:4].view(torch.int32)[0]) == 0, "an activated expert was not resident"
            err = (y_off - y_ref).abs().max().item() / y_ref.abs().max().item()
            assert err < 1e-5, (step, l, err)          # same kernels, same data; only atomics order differs
            counts = b_off.counts.cpu().numpy()
            pop = b_off.pred_pop.cpu().numpy()
            ids = [e for e in range(E) if counts[e] > 0]
            pids = [e for e in range(E) if pop[e] > 0] if l + 1 < L else []
            r = sim.step(l, ids, [int(counts[e]) for e in ids], pids, [int(pop[e]) for e in pids])
            tl, order, loads = off.trace[ntr]
            assert tl == l and order == r.compute_order and loads == r.loads
            hits += len(r.hit_cache) + len(r.hit_prefetch)
            misses += len(r.miss)
            h = chain_next_hidden(h, y_off)
    s = off.stats
    assert s["hit_cache"] + s["hit_prefetch"] == hits and s["miss"] == misses
    assert off.bytes_copied() == (s["miss"] + s["prefetch"]) * off.slot_bytes
    if cache_total >= L * E:
        assert misses == 0
    off.close()


def _offload_case(cfg, L, cache_total, L_shallow, n_max, N, steps, check_steps):
    """Offloaded stack at a model's real expert size: decisions against the cache oracle on every
    step, y against the FFN oracle (fed by the oracle's own routing) on the first `check_steps`
    steps.  No device-wide synchronisation inside a step: the copy streams keep their backlog
    while the next layers run, and y of every layer is compared after the step."""
    from oracle import moe as O
    from workloads import gen_expert
    from helpers import bias_np, f32, ffn_rel_err, oracle_expert
    E = cfg.E
    staging = 2 * E + n_max
    off = OffloadedStack(cfg, cache_total, n_max, staging, DEV, layers=L, L_shallow=L_shallow)
    off.keep_trace = True
    sim = OC.CacheOracle(L, E, cache_total, L_shallow, n_max, staging)
    assert off.caps == sim.caps and off.total_slots == sim.total_slots
    print(f"{cfg.name}: {L} layers, capacities {off.caps}, slot {off.slot_bytes / 1e6:.2f} MB, n_max {n_max}", flush=True)
    buf = LayerBuffers(cfg, N, DEV)
    worst = 0.0
    loads_total = 0
    for step in range(steps):
        h = gen_hidden(cfg, N, step=step, device=DEV).float()
        kept = []
        for l in range(L):
            x = unit_rmsnorm_bf16(h)
            ntr = len(off.trace)
            y = off.layer(l, x, buf)
            status = buf.ffn_ws[:4].view(torch.int32).clone()
            kept.append((x, buf.ids.clone(), buf.w.clone(), buf.counts.clone(), buf.pred_pop.clone(), y.clone(),
                         status, off.trace[ntr]))
            h = chain_next_hidden(h, y)
        torch.cuda.current_stream().synchronize()
        for l, (x, ids, w, counts, pop, y, status, (tl, order, loads)) in enumerate(kept):
            assert int(status[0]) == 0, "an activated expert was not resident"
            counts, pop = counts.cpu().numpy(), pop.cpu().numpy()
            aids = [e for e in range(E) if counts[e] > 0]
            pids = [e for e in range(E) if pop[e] > 0] if l + 1 < L else []
            r = sim.step(l, aids, [int(counts[e]) for e in aids], pids, [int(pop[e]) for e in pids])
            assert tl == l and order == r.compute_order and loads == r.loads, (step, l)
            loads_total += len(loads)
            if step < check_steps:
                Wg, bias = off.gates[l]
                rid, rw, _, rz = O.gate_route(f32(x), f32(Wg), bias_np(bias), cfg.k, cfg.renorm)
                assert len(O.near_tie_rows(rz, cfg.k)) == 0
                assert np.array_equal(ids.cpu().numpy(), rid)
                experts = {int(e): oracle_expert(gen_expert(cfg, l, int(e), device=DEV)) for e in set(rid.ravel().tolist())}
                shared = [oracle_expert(gen_expert(cfg, l, s, shared=True, device=DEV)) for s in range(cfg.n_shared)]
                sg = None if off.shared_gates[l] is None else f32(off.shared_gates[l])
                y_ref = O.moe_ffn(f32(x), rid, rw, experts, shared, sg)
                err = ffn_rel_err(f32(y), y_ref).max()
                worst = max(worst, err)
                assert err <= 2e-3, (step, l, err)
        print(f"  step {step}: decisions equal the cache oracle's; worst FFN row error so far {worst:.2e}", flush=True)
    torch.cuda.synchronize()
    s = off.stats
    assert off.bytes_copied() == loads_total * off.slot_bytes == (s["miss"] + s["prefetch"]) * off.slot_bytes
    assert s["miss"] > 0 and s["hit_cache"] > 0
    off.close()


def test_offloaded_deepseek_shape_against_both_oracles():
    """configs[3] geometry on five layers: one fully cached shallow layer and four deep layers with the
    14 / 13 slots the 30 % budget gives the real 28-layer stack; 4.46 MB experts, batch 8."""
    cfg = SHAPES["deepseek"]
    _offload_case(cfg, L=5, cache_total=64 + 14 + 14 + 13 + 13, L_shallow=1, n_max=8, N=8, steps=5, check_steps=2)


def test_offloaded_mixtral_shape_against_both_oracles():
    """configs[4] geometry on three layers: 90.8 MB experts, one shallow layer full and two of eight
    experts cached in each deep layer (25 %), batch 1."""
    cfg = SHAPES["mixtral"]
    _offload_case(cfg, L=3, cache_total=8 + 2 + 2, L_shallow=1, n_max=1, N=1, steps=6, check_steps=2)


@pytest.mark.parametrize("predictor", ["eap", "none"])
def test_offloaded_stack_comparison_modes(predictor):
    """The baseline modes of section 5.1 on the device: the activation-path predictor (statistics learned
    on the first steps, then used) and no prediction at all feed the same cache step; decisions equal the
    cache oracle fed by the Python predictor, outputs equal the all-resident path."""
    cfg = dataclasses.replace(SHAPES["tiny"], name="tiny4", layers=4)
    L, E, N, n_max, cache_total = cfg.layers, cfg.E, 3, 2, 10
    staging = 2 * E + n_max
    ref = MoEStack(cfg, DEV)
    off = OffloadedStack(cfg, cache_total, n_max, staging, DEV, L_shallow=1, predictor=predictor)
    off.keep_trace = True
    sim = OC.CacheOracle(L, E, cache_total, 1, n_max, staging)
    eap = OC.EAPPredictor(L, E)
    b_ref, b_off = LayerBuffers(cfg, N, DEV), LayerBuffers(cfg, N, DEV)
    prefetched = 0
    for step in range(10):
        learning = step < 5
        off.eap_learning = learning
        h = gen_hidden(cfg, N, step=step, device=DEV).float()
        prev_ids = None
        for l in range(L):
            x = unit_rmsnorm_bf16(h)
            y_ref = layer_forward(cfg, ref.layers[l], ref.layers[l + 1] if l + 1 < L else None, x, b_ref).clone()
            ntr = len(off.trace)
            y_off = off.layer(l, x, b_off)
            torch.cuda.synchronize()
            assert int(b_off.ffn_ws[:4].view(torch.int32)[0]) == 0
            assert (y_off - y_ref).abs().max().item() / y_ref.abs().max().item() < 1e-5
            ids = b_off.ids.cpu().numpy().tolist()
            if predictor == "eap" and learning and prev_ids is not None:
                eap.update(l - 1, prev_ids, ids)
            prev_ids = ids
            counts = b_off.counts.cpu().numpy()
            aids = [e for e in range(E) if counts[e] > 0]
            pop = eap.predict(l, ids, cfg.m) if predictor == "eap" else [0] * E
            pids = [e for e in range(E) if pop[e] > 0] if l + 1 < L else []
            r = sim.step(l, aids, [int(counts[e]) for e in aids], pids, [int(pop[e]) for e in pids])
            tl, order, loads = off.trace[ntr]
            assert tl == l and order == r.compute_order and loads == r.loads, (step, l)
            prefetched += sum(1 for ld in loads if not ld[3])
            h = chain_next_hidden(h, y_off)
    assert (prefetched > 0) == (predictor == "eap")
    off.close()


def test_offloaded_prefill_with_hybrid_transfer_width():
    """Section 4.5 end to end on the device: in a prefill pass the least popular quarter of the predicted
    experts arrives as 2-bit copies.  The load list (experts, slots, widths) equals the cache oracle's, the
    bytes moved are the sum of the copies' sizes, and y equals the FFN oracle evaluated on the copy of every
    expert that the layer really used."""
    from oracle import moe as O
    from workloads import gen_expert
    from helpers import bias_np, f32, ffn_rel_err, oracle_expert
    cfg = dataclasses.replace(SHAPES["qwen_prefill"], layers=3)
    L, E, N = 3, cfg.E, 192
    cache_total, n_max, staging = 60 + 12 + 12, E, 2 * E + E          # layer 0 full, 12 slots in each deep layer
    off = OffloadedStack(cfg, cache_total, n_max, staging, DEV, layers=L, L_shallow=1, low_bits=2)
    off.set_low_percent(25)
    off.keep_trace = True
    sim = OC.CacheOracle(L, E, cache_total, 1, n_max, staging, low_percent=25, bits=4, low_bits=2)
    assert off.caps == sim.caps == [60, 12, 12]
    buf = LayerBuffers(cfg, N, DEV, mode=2)
    width = {}                     # (layer, expert) -> width of the copy staged for it
    n_low = bytes_expected = 0
    h = gen_hidden(cfg, N, step=0, device=DEV).float()
    for l in range(L):
        x = unit_rmsnorm_bf16(h)
        y = off.layer(l, x, buf)
        torch.cuda.synchronize()
        assert int(buf.ffn_ws[:4].view(torch.int32)[0]) == 0
        counts, pop = buf.counts.cpu().numpy(), buf.pred_pop.cpu().numpy()
        aids = [e for e in range(E) if counts[e] > 0]
        pids = [e for e in range(E) if pop[e] > 0] if l + 1 < L else []
        r = sim.step(l, aids, [int(counts[e]) for e in aids], pids, [int(pop[e]) for e in pids])
        tl, order, loads = off.trace[-1]
        assert tl == l and order == r.compute_order and loads == r.loads and off.trace_bits[-1] == r.load_bits
        for (ll, e, _, _), b in zip(r.loads, r.load_bits):
            width[(ll, e)] = b
            n_low += b == 2
            bytes_expected += off.low_slot_bytes if b == 2 else off.slot_bytes
        Wg, bias = off.gates[l]
        rid, rw, _, rz = O.gate_route(f32(x), f32(Wg), bias_np(bias), cfg.k, cfg.renorm)
        ties = set(O.near_tie_rows(rz, cfg.k).tolist())
        rows = [t for t in range(N) if t not in ties]
        assert np.array_equal(buf.ids.cpu().numpy()[rows], rid[rows])
        used = sorted(set(rid.ravel().tolist()))
        experts = {e: oracle_expert(gen_expert(cfg, l, e, device=DEV, bits=width.get((l, e), 4))) for e in used}
        shared = [oracle_expert(gen_expert(cfg, l, s, shared=True, device=DEV)) for s in range(cfg.n_shared)]
        y_ref = O.moe_ffn_grouped(f32(x), rid, rw, experts, shared, f32(off.shared_gates[l]))
        err = ffn_rel_err(f32(y)[rows], y_ref[rows]).max()
        low_used = sorted(e for e in used if width.get((l, e), 4) == 2)
        print(f"layer {l}: {len(used)} experts activated, {len(low_used)} of them from 2-bit copies, max row error "
              f"{err:.2e}", flush=True)
        assert err <= 2e-3
        h = chain_next_hidden(h, y)
    assert n_low > 0 and off.bytes_copied() == bytes_expected
    off.close()


def test_prefill_compute_follows_the_order_of_the_transfers():
    """Section 4.3, figure "rearranging the order of expert computations": experts 2 and 4 are already on
    the device, 3, 1 and 5 are being loaded in that order; the computation runs 2, 4 first and then 3, 1, 5
    as they arrive.  Here on the device path: a layer whose cache holds {2, 4}, tokens routed so that the
    demand loads come out in the order 3, 1, 5, the FFN taken in pieces of one expert."""
    from oracle import moe as O
    from helpers import f32, ffn_rel_err, oracle_expert, gpu_permute
    from workloads import gen_expert
    cfg = dataclasses.replace(SHAPES["tiny"], name="tiny1", layers=1, E=8, k=1, bits=4, group=128)
    E, N = cfg.E, 40
    # the cache preloads experts 0 .. c-1, so the figure's expert ids are renamed: cached {0, 1} play {2, 4},
    # and the loads 5, 3, 7 (by decreasing token count) play 3, 1, 5
    off = OffloadedStack(cfg, cache_total=2, n_max=0, staging_slots=2 * E, device=DEV, layers=1, L_shallow=0)
    off.overlap_piece = 1
    off.keep_trace = True
    assert off.caps == [2]
    x = gen_hidden(cfg, N, device=DEV)
    ids = torch.tensor([[0]] * 6 + [[1]] * 5 + [[5]] * 12 + [[3]] * 9 + [[7]] * 8, dtype=torch.int32, device=DEV)
    w = torch.rand(N, 1, device=DEV) + 0.5
    # drive the stack's layer call with a fixed routing: the routing entry points are replaced by copies
    buf = LayerBuffers(cfg, N, DEV, mode=2)
    import paper_2502_12224_amd.binding as B
    assert not buf.fused_ok              # 40 tokens: the stack calls fate_gate_route and fate_permute
    real = B.fate_gate_route

    def fixed(xx, Wg, bias, k, renorm, oid, ow, probs, stream=None):
        oid.copy_(ids)
        ow.copy_(w)
    B.fate_gate_route = fixed
    try:
        y = off.layer(0, x, buf).clone()
    finally:
        B.fate_gate_route = real
    torch.cuda.synchronize()
    assert int(buf.ffn_ws[:4].view(torch.int32)[0]) == 0
    tl, order, loads = off.trace[-1]
    assert order == [0, 1, 5, 3, 7]                                   # on the device first, then in load order
    assert [(e, d) for (_, e, _, d) in loads] == [(5, True), (3, True), (7, True)]
    assert off.piece_log[-1] == (0, [[0, 1], [5], [3], [7]])
    sim = OC.CacheOracle(1, E, 2, 0, 0, 2 * E)
    r = sim.step(0, [0, 1, 3, 5, 7], [6, 5, 9, 12, 8])
    assert r.compute_order == order and r.loads == loads
    experts = {e: oracle_expert(gen_expert(cfg, 0, e, device=DEV)) for e in (0, 1, 3, 5, 7)}
    y_ref = O.moe_ffn_grouped(f32(x), ids.cpu().numpy(), w.cpu().numpy().astype(np.float64), experts)
    assert ffn_rel_err(f32(y), y_ref).max() <= 2e-3
    # the pieces add up to exactly what one call gives
    g = gpu_permute(ids, E)
    y_one = torch.empty_like(y)
    B.fate_moe_ffn_q(buf.desc, x, off.table_for(0), *g, w, None, None, y_one, buf.ffn_ws)
    torch.cuda.synchronize()
    assert torch.equal(y_one, y)
    off.close()
