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
