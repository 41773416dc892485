"""End-to-end parity at the sizes the benchmark runs: the oracle routes (fp64),
the oracle computes the FFN of the whole layer from its own routing, and the
GPU's routing outputs and y are compared with that - nothing the GPU produced
is handed to the oracle.  Rows whose oracle logits have a top-k gap below 1e-5
are counted apart (their expert set may legitimately differ, and so may y).

FFN bar: per token row max_i |y_gpu - y_ref| / max_i |y_ref| <= 2e-3."""
import time
from types import SimpleNamespace

import numpy as np
import pytest
import torch

from oracle import moe as O
import paper_2502_12224_amd.binding as B
from paper_2502_12224_amd.stack import LayerBuffers, LayerWeights, layer_forward
from workloads import SHAPES, gen_expert, gen_gate, gen_hidden
from helpers import DEV, GpuLayer, bias_np, f32, ffn_rel_err, gpu_permute, gpu_predict, gpu_route, oracle_expert

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _say(msg):
    print(msg, flush=True)


def _oracle_layer(cfg, layer, x, ids, w, grouped=True):
    """Oracle FFN of a whole layer from the oracle's own routing; experts are dequantised one at
    a time (a Mixtral-shaped expert is 1.4 GB in fp64)."""
    xn = f32(x)
    used = sorted(set(ids.ravel().tolist()))
    y = np.zeros((xn.shape[0], cfg.H), dtype=np.float64)
    for e in used:
        ex = {e: oracle_expert(gen_expert(cfg, layer, e, device=DEV))}
        mask = ids == e
        rows = np.nonzero(mask.any(axis=1))[0]
        # only the pairs of expert e: one column per row (an expert appears once in a row)
        col = mask[rows].argmax(axis=1)
        ids1 = np.full((len(rows), 1), e, dtype=np.int32)
        w1 = w[rows, col][:, None]
        f = O.moe_ffn_grouped if grouped else O.moe_ffn
        y[rows] += f(xn[rows], ids1, w1, ex)
        del ex
    shared = [oracle_expert(gen_expert(cfg, layer, s, shared=True, device=DEV)) for s in range(cfg.n_shared)]
    if shared:
        from workloads import gen_shared_gate
        sg = gen_shared_gate(cfg, layer, DEV)
        sg = None if sg is None else f32(sg)
        y += O.moe_ffn_grouped(xn, np.zeros((xn.shape[0], 0), dtype=np.int32), np.zeros((xn.shape[0], 0)), {},
                               shared, sg)
    return y


@pytest.mark.parametrize("name,N", [("qwen_prefill", 512), ("qwen_prefill", 2048), ("deepseek", 1024),
                                    ("mixtral", 2048)])
def test_full_prefill_layer_against_oracle_routing_and_ffn(name, N):
    cfg = SHAPES[name]
    t0 = time.time()
    _say(f"case {name} N={N}: routing")
    x = gen_hidden(cfg, N, device=DEV)
    lw = LayerWeights(cfg, 0, DEV)
    Wg1, b1 = gen_gate(cfg, 1, device=DEV)
    buf = LayerBuffers(cfg, N, DEV, mode=2)
    y = layer_forward(cfg, lw, SimpleNamespace(Wg=Wg1, bias=b1), x, buf)         # fate_route_fused (MFMA gate) + MFMA FFN
    torch.cuda.synchronize()
    assert int(buf.ffn_ws[:4].view(torch.int32)[0]) == 0
    _say(f"  GPU layer done ({time.time() - t0:.0f}s); oracle routing")
    rid, rw, _, rz = O.gate_route(f32(x), f32(lw.Wg), bias_np(lw.bias), cfg.k, cfg.renorm)
    pid, _, rpop, pz = O.cross_layer_predict(f32(x), f32(Wg1), bias_np(b1), cfg.m)
    ties = set(O.near_tie_rows(rz, cfg.k).tolist())
    pties = set(O.near_tie_rows(pz, cfg.m).tolist())
    rows = np.array([t for t in range(N) if t not in ties])
    assert len(ties) <= max(1, N // 200) and len(pties) <= max(1, N // 100)
    ids_g = buf.ids.cpu().numpy()
    assert np.array_equal(ids_g[rows], rid[rows])
    assert (np.abs(buf.w.cpu().numpy()[rows] - rw[rows]) <= 1e-6 + 1e-5 * np.abs(rw[rows])).all()
    prow = np.array([t for t in range(N) if t not in pties])
    assert np.array_equal(buf.pred_ids.cpu().numpy()[prow], pid[prow])
    if not pties:
        assert np.array_equal(buf.pred_pop.cpu().numpy(), rpop)
    if not ties:
        for a, r in zip((buf.counts, buf.offsets, buf.perm[:N * cfg.k], buf.inv_perm[:N * cfg.k], buf.order),
                        O.permute(rid, cfg.E)):
            assert np.array_equal(a.cpu().numpy(), r)
    else:   # the permutation of the GPU's own ids (those differ from the oracle's only in near-tie rows)
        for a, r in zip((buf.counts, buf.offsets, buf.perm[:N * cfg.k], buf.inv_perm[:N * cfg.k], buf.order),
                        O.permute(ids_g, cfg.E)):
            assert np.array_equal(a.cpu().numpy(), r)
    _say(f"  routing exact on {len(rows)} rows, {len(ties)} near-tie rows apart ({time.time() - t0:.0f}s); oracle FFN "
         f"of the whole layer ({len(set(rid.ravel().tolist()))} experts + {cfg.n_shared} shared)")
    del lw
    torch.cuda.empty_cache()
    y_ref = _oracle_layer(cfg, 0, x, rid, rw)
    err = ffn_rel_err(f32(y)[rows], y_ref[rows])
    counts = np.bincount(rid.ravel(), minlength=cfg.E)
    _say(f"  max row error {err.max():.2e} over {len(rows)} rows; expert rows min/max {counts.min()}/{counts.max()} "
         f"({time.time() - t0:.0f}s)")
    assert np.isfinite(f32(y)).all() and err.max() <= TOL


def test_prefill_segment_edges_against_the_pairwise_oracle():
    """Qwen-shaped prefill, 512 tokens: for every activated expert the first and last row of its
    segment and the rows on both sides of every 64-row tile edge inside it, and the same rows of
    the shared expert's segment (all tokens), against the pair-by-pair definition."""
    cfg = SHAPES["qwen_prefill"]
    N = 512
    x = gen_hidden(cfg, N, device=DEV)
    Wg, b = gen_gate(cfg, 0, device=DEV)
    rid, rw, _, rz = O.gate_route(f32(x), f32(Wg), bias_np(b), cfg.k, cfg.renorm)
    ties = set(O.near_tie_rows(rz, cfg.k).tolist())
    counts, offsets, perm, inv, order = O.permute(rid, cfg.E)
    want = set()
    for e in range(cfg.E):
        c = int(counts[e])
        pos = {0, c - 1} | {p for edge in range(64, c, 64) for p in (edge - 1, edge)} if c else set()
        want |= {int(perm[offsets[e] + p]) // cfg.k for p in pos}
    want |= {0, N - 1} | {p for edge in range(64, N, 64) for p in (edge - 1, edge)}
    rows = sorted(want - ties)
    ids_d = torch.from_numpy(rid).to(DEV)
    w_d = torch.from_numpy(rw.astype(np.float32)).to(DEV)
    g = gpu_permute(ids_d, cfg.E)
    L = GpuLayer(cfg, 0)
    y, ws = L.ffn(x, *g, w_d, mode=2)
    assert int(ws[:4].view(torch.int32)[0]) == 0
    _say(f"segment edges: {len(rows)} token rows, {int((counts > 0).sum())} activated experts, "
         f"smallest segment {int(counts[counts > 0].min())} rows, largest {int(counts.max())}")
    need = sorted(set(rid[rows].ravel().tolist()))
    experts = {e: oracle_expert(L.host[e]) for e in need}
    shared = [oracle_expert(ex) for ex in L.shared_host]
    y_ref = O.moe_ffn_rows(f32(x), rid, w_d.cpu().numpy().astype(np.float64), experts, shared, f32(L.shared_gate),
                           rows=rows)
    err = ffn_rel_err(f32(y)[rows], y_ref)
    _say(f"  max row error {err.max():.2e}")
    assert err.max() <= TOL


@pytest.mark.parametrize("name,N", [("deepseek", 8), ("mixtral", 1)])
def test_one_launch_decode_layer_end_to_end_against_oracle(name, N):
    """fate_moe_layer_decode (the looping kernels on these two shapes) against oracle routing ->
    oracle prediction -> oracle permutation -> oracle FFN."""
    cfg = SHAPES[name]
    _say(f"case {name} N={N}")
    x = gen_hidden(cfg, N, step=5, device=DEV)
    lw = LayerWeights(cfg, 0, DEV)
    ln = LayerWeights(cfg, 1, DEV, experts=[])
    buf = LayerBuffers(cfg, N, DEV)
    assert buf.one_launch_ok
    y = layer_forward(cfg, lw, ln, x, buf, one_launch=True)
    torch.cuda.synchronize()
    assert buf.status() == 0
    rid, rw, _, rz = O.gate_route(f32(x), f32(lw.Wg), bias_np(lw.bias), cfg.k, cfg.renorm)
    pid, pw, pop, pz = O.cross_layer_predict(f32(x), f32(ln.Wg), bias_np(ln.bias), cfg.m)
    assert len(O.near_tie_rows(rz, cfg.k)) == 0 and len(O.near_tie_rows(pz, cfg.m)) == 0
    assert np.array_equal(buf.ids.cpu().numpy(), rid) and np.array_equal(buf.pred_ids.cpu().numpy(), pid)
    assert np.array_equal(buf.pred_pop.cpu().numpy(), pop)
    assert np.abs(buf.w.cpu().numpy() - rw).max() <= 1e-6 and np.abs(buf.pred_w.cpu().numpy() - pw).max() <= 1e-6
    P = N * cfg.k
    for a, r in zip((buf.counts, buf.offsets, buf.perm[:P], buf.inv_perm[:P], buf.order), O.permute(rid, cfg.E)):
        assert np.array_equal(a.cpu().numpy(), r)
    y_ref = _oracle_layer(cfg, 0, x, rid, rw, grouped=False)
    err = ffn_rel_err(f32(y), y_ref).max()
    _say(f"  max row error {err:.2e}")
    assert err <= TOL


def _expected_with_duplicated_rows(z_even, width):
    """Experts 2j and 2j+1 have the same logit: the selection of `width` experts is the ranking of
    the distinct values with every j expanded to (2j, 2j+1), the lower id first."""
    N = z_even.shape[0]
    out = np.empty((N, width), dtype=np.int32)
    for t in range(N):
        order = sorted(range(z_even.shape[1]), key=lambda j: (-z_even[t, j], j))
        flat = [e for j in order for e in (2 * j, 2 * j + 1)]
        out[t] = flat[:width]
    return out


def test_exact_logit_ties_go_to_the_lower_expert_id():
    """Duplicated gate rows give bit-identical logits: every selection among equals must take
    the lower id, in all routing entry points (row kernel, matrix-core gate, one-launch layer)."""
    cfg = SHAPES["qwen"]
    E, k, m, H = cfg.E, cfg.k, cfg.m, cfg.H
    for N in (1, 7, 300):
        x = gen_hidden(cfg, N, device=DEV)
        Wg, _ = gen_gate(cfg, 0, device=DEV)
        Wg = Wg.clone()
        for e in range(1, E, 2):          # experts 2j and 2j+1 share a gate row (and no bias)
            Wg[e] = Wg[e - 1]
        ids, w, probs = gpu_route(x, Wg, None, k, False)
        pid, pw, pop = gpu_predict(x, Wg, None, k, m)
        torch.cuda.synchronize()
        z_even = O.gate_logits(f32(x), f32(Wg)[0::2])
        # rows where two distinct values are closer than the margin are set apart as usual
        ties = set(O.near_tie_rows(z_even, m // 2 + 1).tolist())
        rows = [t for t in range(N) if t not in ties]
        assert len(rows) >= N - 2
        assert np.array_equal(ids.cpu().numpy()[rows], _expected_with_duplicated_rows(z_even, k)[rows]), N
        assert np.array_equal(pid.cpu().numpy()[rows], _expected_with_duplicated_rows(z_even, m)[rows]), N
        probs = probs.cpu().numpy()
        assert np.array_equal(probs[:, 0::2], probs[:, 1::2])          # the GPU's logits of equal rows are equal bits
        rid, _, _, rz = O.gate_route(f32(x), f32(Wg), None, k, False)
        if (rz[:, 0::2] == rz[:, 1::2]).all():                         # (the host BLAS need not give equal bits)
            assert np.array_equal(ids.cpu().numpy()[rows], rid[rows]), N
    # the one-launch decode layer takes the same decisions
    N = 4
    x = gen_hidden(cfg, N, device=DEV)
    lw = LayerWeights(cfg, 0, DEV)
    for e in range(1, E, 2):
        lw.Wg[e] = lw.Wg[e - 1]
    lw.bias = None
    buf = LayerBuffers(cfg, N, DEV)
    layer_forward(cfg, lw, None, x, buf, one_launch=True)
    torch.cuda.synchronize()
    z_even = O.gate_logits(f32(x), f32(lw.Wg)[0::2])
    assert len(O.near_tie_rows(z_even, k // 2 + 1)) == 0
    assert buf.status() == 0 and np.array_equal(buf.ids.cpu().numpy(), _expected_with_duplicated_rows(z_even, k))


@pytest.mark.parametrize("name,N", [("tiny", 16), ("mixtral", 3), ("tiny", 100)])
def test_selection_of_every_expert(name, N):
    """k = E and m = E: the selection returns all experts, ordered by logit."""
    cfg = SHAPES[name]
    E = cfg.E
    x = gen_hidden(cfg, N, device=DEV)
    Wg, b = gen_gate(cfg, 0, device=DEV)
    ids, w, _ = gpu_route(x, Wg, b, E, True)
    pid, pw, pop = gpu_predict(x, Wg, b, E, E)
    torch.cuda.synchronize()
    rid, rw, _, rz = O.gate_route(f32(x), f32(Wg), bias_np(b), E, True)
    ties = set(O.near_tie_rows(rz, E).tolist())
    rows = [t for t in range(N) if t not in ties]
    assert len(ties) <= 1
    assert np.array_equal(ids.cpu().numpy()[rows], rid[rows]) and np.array_equal(pid.cpu().numpy()[rows], rid[rows])
    assert np.abs(w.cpu().numpy() - rw)[rows].max() <= 1e-6
    assert (np.sort(ids.cpu().numpy(), axis=1) == np.arange(E)[None, :]).all()
    assert pop.cpu().numpy().tolist() == [N] * E
    counts, offsets, perm, inv, order = gpu_permute(ids, E)
    assert counts.cpu().numpy().tolist() == [N] * E and order.cpu().numpy().tolist() == list(range(E))


@pytest.mark.parametrize("name,N", [("qwen", 96), ("tiny", 70)])
def test_mfma_ffn_with_offset_and_outlier_activations(name, N):
    """The matrix-core FFN keeps x, h and the per-pair outputs in fp16: activations with a common
    offset and a few 40x outlier channels (still far inside the fp16 range) must stay within the bar."""
    cfg = SHAPES[name]
    g = torch.Generator(device="cpu").manual_seed(99 + N)
    xf = torch.randn(N, cfg.H, generator=g) + 3.0
    cols = torch.randperm(cfg.H, generator=g)[:8]
    xf[:, cols] *= 40.0
    x = xf.to(torch.bfloat16).to(DEV)
    Wg, b = gen_gate(cfg, 0, device=DEV)
    rid, rw, _, rz = O.gate_route(f32(x), f32(Wg), bias_np(b), cfg.k, cfg.renorm)
    ids_d = torch.from_numpy(rid).to(DEV)
    w_d = torch.from_numpy(rw.astype(np.float32)).to(DEV)
    L = GpuLayer(cfg, 0, experts=sorted(set(rid.ravel().tolist())))
    y, ws = L.ffn(x, *gpu_permute(ids_d, cfg.E), w_d, mode=2)
    assert int(ws[:4].view(torch.int32)[0]) == 0
    experts = {e: oracle_expert(L.host[e]) for e in L.host}
    shared = [oracle_expert(ex) for ex in L.shared_host]
    sg = None if L.shared_gate is None else f32(L.shared_gate)
    y_ref = O.moe_ffn_grouped(f32(x), rid, w_d.cpu().numpy().astype(np.float64), experts, shared, sg)
    err = ffn_rel_err(f32(y), y_ref)
    _say(f"{name} N={N} outliers: max row error {err.max():.2e}")
    assert np.isfinite(f32(y)).all() and err.max() <= TOL
