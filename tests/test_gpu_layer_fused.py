"""One-launch decode layer against the separate calls and the oracle."""
import numpy as np
import pytest
import torch

from oracle import moe as O
import paper_2502_12224_amd.binding as B
from paper_2502_12224_amd.stack import LayerBuffers, LayerWeights, layer_forward
from workloads import SHAPES, gen_hidden
from helpers import DEV, bias_np, f32, ffn_rel_err, oracle_expert

pytestmark = pytest.mark.gpu

ROUTE_FIELDS = ("ids", "w", "counts", "offsets", "perm", "inv_perm", "order")
PRED_FIELDS = ("pred_ids", "pred_w", "pred_pop")


def _snapshot(buf, fields):
    return {f: getattr(buf, f).clone() for f in fields}


@pytest.mark.parametrize("name,N,last", [("tiny", 1, False), ("tiny", 8, False), ("tiny", 5, True),
                                         ("qwen", 1, False), ("qwen", 1, True), ("qwen", 6, False),
                                         ("deepseek", 8, False), ("deepseek", 1, False), ("mixtral", 1, False),
                                         ("mixtral", 4, False)])
def test_one_launch_layer_equals_separate_calls_and_oracle(name, N, last):
    _one_launch_case(SHAPES[name], name, N, last)


# the other kernel instantiations of the one-token form, and a layer without shared experts: the Qwen shape with
# 8-bit routed experts, with an 8-bit shared expert, with both, and with no shared expert at all
import dataclasses
_QWEN = SHAPES["qwen"]
VARIANTS = {
    "qwen-routed8": dataclasses.replace(_QWEN, name="qwen-routed8", bits=8),
    "qwen-shared8": dataclasses.replace(_QWEN, name="qwen-shared8", shared_bits=8),
    "qwen-both8": dataclasses.replace(_QWEN, name="qwen-both8", bits=8, shared_bits=8),
    "qwen-noshared": dataclasses.replace(_QWEN, name="qwen-noshared", n_shared=0, I_shared=0, shared_gate=False),
}


@pytest.mark.parametrize("name,N", [("qwen-routed8", 1), ("qwen-shared8", 1), ("qwen-both8", 1), ("qwen-noshared", 1),
                                    ("qwen-noshared", 3)])
def test_one_launch_layer_on_other_formats_and_without_shared_experts(name, N):
    _one_launch_case(VARIANTS[name], name, N, False)


def _one_launch_case(cfg, name, N, last):
    print(f"case {name} N={N} last={last}", flush=True)
    x = gen_hidden(cfg, N, device=DEV)
    lw = LayerWeights(cfg, 0, DEV)
    ln = None
    if not last:
        ln = LayerWeights(cfg, 1, DEV, experts=[])
    sep = LayerBuffers(cfg, N, DEV)
    one = LayerBuffers(cfg, N, DEV)
    assert one.one_launch_ok
    layer_forward(cfg, lw, ln, x, sep, one_launch=False)
    torch.cuda.synchronize()
    y_sep = sep.y.clone()
    fields = ROUTE_FIELDS + (() if last else PRED_FIELDS)
    want = _snapshot(sep, fields)
    P = N * cfg.k
    # three calls in a row on the same workspace: the counters must come back to zero each time
    for rep in range(3):
        one.y.fill_(float("nan"))
        layer_forward(cfg, lw, ln, x, one, one_launch=True)
        torch.cuda.synchronize()
        assert one.status() == 0, f"status {one.status()} on call {rep}"
        for f in fields:
            a, b = getattr(one, f), want[f]
            if f in ("perm", "inv_perm"):
                a, b = a[:P], b[:P]
            assert torch.equal(a, b), (f, rep)
        y_one = f32(one.y)
        assert np.isfinite(y_one).all()
        # same weights and activations; the two paths differ in the order of the fp32 sums and in how
        # the codes' offset is removed (per code, or per group after the matrix cores), which can
        # move an fp16 rounding of h
        assert ffn_rel_err(y_one, f32(y_sep).astype(np.float64)).max() <= 5e-4, rep
    sync_words = one.layer_ws[:8].view(torch.int32).cpu().numpy()
    assert sync_words[0] == 3 and sync_words[1] == 0       # epoch = number of calls, exit counter back at zero
    # against the oracle
    rid, rw, _, rz = O.gate_route(f32(x), f32(lw.Wg), bias_np(lw.bias), cfg.k, cfg.renorm)
    if len(O.near_tie_rows(rz, cfg.k)) == 0:
        assert np.array_equal(one.ids.cpu().numpy(), rid)
    ids_h = one.ids.cpu().numpy()
    from workloads import gen_expert
    experts = {int(e): oracle_expert(gen_expert(cfg, 0, int(e), device=DEV)) for e in set(ids_h.ravel().tolist())}
    shared = [oracle_expert(gen_expert(cfg, 0, s, shared=True, device=DEV)) for s in range(cfg.n_shared)]
    sg = None if lw.shared_gate is None else f32(lw.shared_gate)
    y_ref = O.moe_ffn(f32(x), ids_h, one.w.cpu().numpy().astype(np.float64), experts, shared, sg)
    err = ffn_rel_err(f32(one.y), y_ref).max()
    print(f"  max row error vs oracle {err:.2e}")
    assert err <= 2e-3


def test_one_launch_layer_rejects_large_batches():
    cfg = SHAPES["tiny"]
    d = B.make_ffn_desc(9, cfg.H, cfg.E, cfg.k, cfg.I, cfg.bits, cfg.group, 0, 0, cfg.bits, cfg.group, True, 0)
    nbytes, _ = B.fate_moe_layer_decode_workspace(d)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    buf = LayerBuffers(cfg, 9, DEV)
    lw = LayerWeights(cfg, 0, DEV)
    x = gen_hidden(cfg, 9, device=DEV)
    with pytest.raises(B.FateError):
        B.fate_moe_layer_decode(d, x, lw.Wg, lw.bias, None, None, cfg.m, cfg.renorm, buf.ids, buf.w, None, None, None,
                                buf.counts, buf.offsets, buf.perm, buf.inv_perm, buf.order, lw.table, None, None,
                                buf.y, ws)

@pytest.mark.parametrize("name,N", [("qwen", 1), ("qwen", 4), ("mixtral", 2)])
def test_one_launch_layer_with_outlier_activations(name, N):
    """Activations with a large common component and a few outlier channels: the one-launch body feeds
    the matrix cores with codes + constant and removes the constant's share afterwards from the sum of
    the activations of a group, which is where such inputs would cost accuracy."""
    cfg = SHAPES[name]
    print(f"case {name} N={N} outliers", flush=True)
    g = torch.Generator(device="cpu").manual_seed(1234 + N)
    xf = torch.randn(N, cfg.H, generator=g) + 3.0                       # common offset: every group sum is large
    cols = torch.randperm(cfg.H, generator=g)[:8]
    xf[:, cols] *= 40.0                                                  # outlier channels
    x = xf.to(torch.bfloat16).to(DEV)
    lw = LayerWeights(cfg, 0, DEV)
    one = LayerBuffers(cfg, N, DEV)
    layer_forward(cfg, lw, None, x, one, one_launch=True)
    torch.cuda.synchronize()
    assert one.status() == 0
    ids_h = one.ids.cpu().numpy()
    from workloads import gen_expert
    experts = {int(e): oracle_expert(gen_expert(cfg, 0, int(e), device=DEV)) for e in set(ids_h.ravel().tolist())}
    shared = [oracle_expert(gen_expert(cfg, 0, s, shared=True, device=DEV)) for s in range(cfg.n_shared)]
    sg = None if lw.shared_gate is None else f32(lw.shared_gate)
    y_ref = O.moe_ffn(f32(x), ids_h, one.w.cpu().numpy().astype(np.float64), experts, shared, sg)
    err = ffn_rel_err(f32(one.y), y_ref).max()
    print(f"  max row error vs oracle {err:.2e}")
    assert err <= 2e-3

@pytest.mark.parametrize("name,N,how", [("qwen", 1, "null"), ("qwen", 6, "null"), ("mixtral", 1, "null"),
                                        ("qwen", 1, "zero_points"), ("qwen", 6, "zero_points")])
def test_one_launch_layer_with_an_expert_that_is_not_resident(name, N, how):
    """An activated expert whose table entry holds NULL pointers, or is stored in a format the one-launch
    layer does not read (here: with zero-points): status bit 0 is raised, its pairs contribute nothing,
    everything else is as usual (one-item and looping kernels)."""
    cfg = SHAPES[name]
    print(f"case {name} N={N} one expert absent ({how})", flush=True)
    x = gen_hidden(cfg, N, device=DEV)
    lw = LayerWeights(cfg, 0, DEV)
    one = LayerBuffers(cfg, N, DEV)
    layer_forward(cfg, lw, None, x, one, one_launch=True)
    torch.cuda.synchronize()
    ids_h = one.ids.cpu().numpy()
    gone = int(ids_h[0, 0])                                  # the first token's first expert
    saved = lw.table.clone()
    sz = __import__('ctypes').sizeof(B.fate_qexpert)
    if how == "null":
        lw.table[gone * sz:(gone + 1) * sz].zero_()
    else:                      # a non-NULL zero-point pointer (the scales' address: never read)
        o = B.fate_qexpert
        lw.table[gone * sz + o.z1.offset:gone * sz + o.z1.offset + 8] = \
            lw.table[gone * sz + o.s1.offset:gone * sz + o.s1.offset + 8].clone()
    one.y.fill_(float("nan"))
    layer_forward(cfg, lw, None, x, one, one_launch=True)
    torch.cuda.synchronize()
    lw.table.copy_(saved)
    assert one.status() == 1
    assert np.array_equal(one.ids.cpu().numpy(), ids_h)
    from workloads import gen_expert
    experts = {int(e): oracle_expert(gen_expert(cfg, 0, int(e), device=DEV)) for e in set(ids_h.ravel().tolist())}
    shared = [oracle_expert(gen_expert(cfg, 0, s, shared=True, device=DEV)) for s in range(cfg.n_shared)]
    sg = None if lw.shared_gate is None else f32(lw.shared_gate)
    w_ref = one.w.cpu().numpy().astype(np.float64)
    w_ref[ids_h == gone] = 0.0
    y_ref = O.moe_ffn(f32(x), ids_h, w_ref, experts, shared, sg)
    err = ffn_rel_err(f32(one.y), y_ref).max()
    print(f"  max row error vs oracle {err:.2e}")
    assert err <= 2e-3


@pytest.mark.parametrize("name,N", [("qwen", 1), ("deepseek", 8)])
def test_one_launch_layer_replayed_from_a_graph(name, N):
    """The layer call captured once and replayed with new inputs, with eager calls and synchronisations
    between the replays: every replay gives what the eager call gives on the same input, bit for bit
    (one-item and looping kernels; the call's epoch lives on the device, so a replay advances it)."""
    cfg = SHAPES[name]
    print(f"case {name} N={N} graph replays", flush=True)
    lw = LayerWeights(cfg, 0, DEV)
    ln = LayerWeights(cfg, 1, DEV, experts=[])
    xs = [gen_hidden(cfg, N, step=s, device=DEV) for s in range(4)]
    eager = LayerBuffers(cfg, N, DEV)
    fields = ROUTE_FIELDS + PRED_FIELDS
    want = []
    for x in xs:
        layer_forward(cfg, lw, ln, x, eager, one_launch=True)
        torch.cuda.synchronize()
        assert eager.status() == 0
        want.append((_snapshot(eager, fields), eager.y.clone()))
    cap = LayerBuffers(cfg, N, DEV)
    x_in = torch.zeros_like(xs[0])
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        x_in.copy_(xs[0])
        layer_forward(cfg, lw, ln, x_in, cap, one_launch=True)     # warm before capture
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            layer_forward(cfg, lw, ln, x_in, cap, one_launch=True)
    torch.cuda.synchronize()
    for s in (1, 3, 0, 2, 2):
        x_in.copy_(xs[s])
        cap.y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert cap.status() == 0
        for f in fields:
            assert torch.equal(getattr(cap, f), want[s][0][f]), f"{f} of a replay (input {s}) differs from the eager call"
        assert torch.equal(cap.y, want[s][1]), f"y of a replay (input {s}) differs from the eager call"
        # eager work of the program between the replays
        layer_forward(cfg, lw, ln, xs[(s + 1) % 4], eager, one_launch=True)
        torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["qwen", "deepseek"])
def test_one_token_layer_with_prefetch_hints(name):
    """The previous layer's prediction handed in as a hint (section 4.3): the routed work groups start on
    the hinted experts before the gate is known.  Whatever the hint - exact, permuted, partly or wholly
    wrong, repeated, out of range, pointing at an expert that is not resident - the routing outputs are
    those of the call without a hint, bit for bit, and y differs at most in the order of its fp32 sums."""
    cfg = SHAPES[name]
    E, k = cfg.E, cfg.k
    x = gen_hidden(cfg, 1, step=11, device=DEV)
    lw = LayerWeights(cfg, 0, DEV)
    ln = LayerWeights(cfg, 1, DEV, experts=[])
    ref = LayerBuffers(cfg, 1, DEV)
    layer_forward(cfg, lw, ln, x, ref, one_launch=True)
    torch.cuda.synchronize()
    assert ref.status() == 0
    true = ref.ids.cpu().numpy()[0].tolist()
    others = [e for e in range(E) if e not in true]
    # an expert that is not selected and not resident: a hint may name it without consequences
    gone = others[0]
    sz = __import__('ctypes').sizeof(B.fate_qexpert)
    lw.table[gone * sz:(gone + 1) * sz].zero_()
    hints = {
        "exact": true,
        "reversed": true[::-1],
        "one wrong": true[:1] + [others[1]] + true[2:],
        "all wrong": others[1:1 + k],
        "repeated": [true[0]] * k,
        "out of range": [-1, E + 5] + true[:k - 2],
        "not resident": [gone] + true[1:],
    }
    y_ref = f32(ref.y).astype(np.float64)
    fields = ROUTE_FIELDS + PRED_FIELDS
    got = LayerBuffers(cfg, 1, DEV)
    for what, h in hints.items():
        print(f"case {name} hint {what}: {h}", flush=True)
        hint = torch.tensor(h, dtype=torch.int32, device=DEV)
        got.y.fill_(float("nan"))
        layer_forward(cfg, lw, ln, x, got, one_launch=True, hint_ids=hint)
        torch.cuda.synchronize()
        assert got.status() == 0, what
        for f in fields:
            assert torch.equal(getattr(got, f), getattr(ref, f)), (what, f)
        assert ffn_rel_err(f32(got.y), y_ref).max() <= 1e-5, what
    # against the oracle once more, with the exact hint
    hint = torch.tensor(true, dtype=torch.int32, device=DEV)
    layer_forward(cfg, lw, ln, x, got, one_launch=True, hint_ids=hint)
    torch.cuda.synchronize()
    from workloads import gen_expert
    experts = {int(e): oracle_expert(gen_expert(cfg, 0, int(e), device=DEV)) for e in true}
    shared = [oracle_expert(gen_expert(cfg, 0, s, shared=True, device=DEV)) for s in range(cfg.n_shared)]
    sg = None if lw.shared_gate is None else f32(lw.shared_gate)
    y_orc = O.moe_ffn(f32(x), ref.ids.cpu().numpy(), ref.w.cpu().numpy().astype(np.float64), experts, shared, sg)
    assert ffn_rel_err(f32(got.y), y_orc).max() <= 2e-3
