"""GPU parity of routing, prediction and permutation against the oracle
(through the C ABI).  Integer outputs must match bit for bit; rows whose
oracle logits have a top-k gap below 1e-5 are counted apart."""
import numpy as np
import pytest
import torch

from oracle import moe as O
import paper_2502_12224_amd.binding as B
from workloads import SHAPES, gen_gate, gen_hidden
from helpers import DEV, bias_np, check_routing, f32, gpu_permute, gpu_predict, gpu_route

pytestmark = pytest.mark.gpu

CASES = [("tiny", 16), ("qwen", 1), ("qwen", 5), ("qwen", 77), ("qwen_prefill", 512), ("qwen_prefill", 2048),
         ("deepseek", 8), ("deepseek", 1024), ("mixtral", 1), ("mixtral", 3), ("mixtral", 300), ("mixtral", 2048)]


@pytest.mark.parametrize("name,N", CASES)
def test_gate_route_matches_oracle(name, N):
    cfg = SHAPES[name]
    x = gen_hidden(cfg, N, device=DEV)
    Wg, b = gen_gate(cfg, 0, device=DEV)
    ids, w, probs = gpu_route(x, Wg, b, cfg.k, cfg.renorm)
    torch.cuda.synchronize()
    rid, rw, rp, rz = O.gate_route(f32(x), f32(Wg), bias_np(b), cfg.k, cfg.renorm)
    nt = check_routing(ids, w, rid, rw, rz, cfg.k, f"{name} N={N}")
    assert nt <= max(1, N // 200)
    p = probs.cpu().numpy().astype(np.float64)
    assert np.abs(p - rp).max() <= 1e-6 and np.allclose(p.sum(1), 1, atol=1e-5)


@pytest.mark.parametrize("name,N", CASES)
def test_cross_layer_predict_matches_oracle(name, N):
    cfg = SHAPES[name]
    x = gen_hidden(cfg, N, device=DEV)
    Wg1, b1 = gen_gate(cfg, 1, device=DEV)
    m = cfg.m
    ids, w, pop = gpu_predict(x, Wg1, b1, cfg.k, m)
    torch.cuda.synchronize()
    rid, rw, rpop, rz = O.cross_layer_predict(f32(x), f32(Wg1), bias_np(b1), m)
    nt = check_routing(ids, w, rid, rw, rz, m, f"{name} N={N}")
    if nt == 0:
        assert np.array_equal(pop.cpu().numpy(), rpop)
    assert int(pop.sum()) == N * m
    # identity: the same gate on the same input is that layer's true routing
    tid, tw, _ = gpu_route(x, Wg1, b1, cfg.k, False, want_probs=False)
    assert torch.equal(tid, ids[:, :cfg.k]) and torch.equal(tw, w[:, :cfg.k])


@pytest.mark.parametrize("N,k,E", [(0, 2, 8), (1, 4, 60), (16, 2, 8), (5, 6, 64), (512, 4, 60), (2048, 6, 64),
                                   (4096, 8, 256), (1000, 1, 3)])
def test_permute_matches_oracle(N, k, E):
    rng = np.random.default_rng(N * 7 + k)
    # skewed draws without repeats inside a row
    pw = 1.0 / np.arange(1, E + 1) ** 1.1
    ids = np.stack([rng.choice(E, size=k, replace=False, p=pw / pw.sum()) for _ in range(N)]).astype(np.int32) \
        if N else np.zeros((0, k), np.int32)
    g = gpu_permute(torch.from_numpy(ids).to(DEV), E)
    torch.cuda.synchronize()
    ref = O.permute(ids, E)
    for a, r, nm in zip(g, ref, ("counts", "offsets", "perm", "inv_perm", "expert_order")):
        assert np.array_equal(a.cpu().numpy(), r), nm


def test_permute_drops_out_of_range_ids():
    ids = torch.tensor([[0, 9], [3, -1], [3, 0]], dtype=torch.int32, device=DEV)
    counts, offsets, perm, inv, order = gpu_permute(ids, 4)
    assert counts.tolist() == [2, 0, 0, 2] and offsets.tolist() == [0, 2, 2, 2, 4]
    assert perm[:4].tolist() == [0, 5, 2, 4] and inv.tolist() == [0, -1, 2, -1, 3, 1]


@pytest.mark.parametrize("name,N", [("tiny", 16), ("qwen", 1), ("qwen", 5), ("deepseek", 8), ("mixtral", 1), ("mixtral", 4),
                                    ("qwen", 512), ("qwen", 2047), ("deepseek", 1024), ("mixtral", 2048)])
def test_route_fused_equals_the_three_calls(name, N):
    cfg = SHAPES[name]
    x = gen_hidden(cfg, N, device=DEV)
    Wg, b = gen_gate(cfg, 0, device=DEV)
    Wg1, b1 = gen_gate(cfg, 1, device=DEV)
    E, k, m = cfg.E, cfg.k, cfg.m
    ws = torch.zeros(B.fate_route_fused_workspace(N, E), dtype=torch.uint8, device=DEV)
    mk = lambda *s, dt=torch.int32: torch.full(s, -3, dtype=dt, device=DEV)
    for rep in range(3):           # the workspace must come back clean
        ids, w = mk(N, k), mk(N, k, dt=torch.float32)
        pid, pw, pop = mk(N, m), mk(N, m, dt=torch.float32), mk(E)
        counts, offsets, perm, inv, order = mk(E), mk(E + 1), mk(N * k), mk(N * k), mk(E)
        B.fate_route_fused(x, Wg, b, Wg1, b1, k, m, cfg.renorm, ids, w, pid, pw, pop, counts, offsets, perm, inv,
                           order, ws)
        torch.cuda.synchronize()
        assert int(ws[:4].view(torch.int32)[0]) == 0
        sid, sw, _ = gpu_route(x, Wg, b, k, cfg.renorm, want_probs=False)
        spid, spw, spop = gpu_predict(x, Wg1, b1, k, m)
        sperm = gpu_permute(sid, E)
        torch.cuda.synchronize()
        for a, r in ((ids, sid), (w, sw), (pid, spid), (pw, spw), (pop, spop), (counts, sperm[0]),
                     (offsets, sperm[1]), (perm, sperm[2]), (inv, sperm[3]), (order, sperm[4])):
            assert torch.equal(a, r)
    # last layer: no next gate
    ids, w = mk(N, k), mk(N, k, dt=torch.float32)
    B.fate_route_fused(x, Wg, b, None, None, k, m, cfg.renorm, ids, w, None, None, None, counts, offsets, perm,
                       inv, order, ws)
    torch.cuda.synchronize()
    assert torch.equal(ids, sid) and torch.equal(w, sw)
