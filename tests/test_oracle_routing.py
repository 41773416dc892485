"""Pins of the routing / prediction / permutation oracle against things other
than itself: scipy's softmax, full sorts, numpy's stable argsort, constructed
ties, and the identity that defines the cross-layer prediction."""
import numpy as np
import pytest
import scipy.special
import torch

from oracle import moe as O
from workloads import SHAPES, gen_hidden, gen_gate, default_m


def _f(t):
    return t.to(torch.float32).numpy()


def test_softmax_matches_scipy_and_sums_to_one():
    rng = np.random.default_rng(0)
    z = rng.normal(size=(37, 60)) * 3
    p = O.softmax(z)
    assert np.allclose(p.sum(axis=1), 1.0, atol=1e-12)
    assert np.allclose(p, scipy.special.softmax(z, axis=1), rtol=1e-13, atol=0)
    # shift invariance and a single expert
    assert np.allclose(O.softmax(z + 123.456), p, rtol=1e-12)
    assert np.all(O.softmax(rng.normal(size=(5, 1))) == 1.0)
    # very large logits do not overflow
    assert np.isfinite(O.softmax(z * 1e3)).all()


def test_gate_logits_is_the_linear_map():
    # a hand-computable case: one-hot rows pick columns of Wg, bias added
    Wg = np.arange(12, dtype=np.float64).reshape(3, 4)       # E=3, H=4
    x = np.eye(4)[[2, 0]]
    b = np.array([0.5, -1.0, 2.0])
    z = O.gate_logits(x, Wg, b)
    assert np.array_equal(z, np.array([[2.5, 5.0, 12.0], [0.5, 3.0, 10.0]]))
    # transposed-operand mistake would fail: x @ Wg (shape mismatch) or Wg @ x


def test_topk_brute_force_and_ties():
    rng = np.random.default_rng(1)
    z = rng.normal(size=(50, 16))
    for k in (1, 2, 6, 16):
        ids = O.topk_ids(z, k)
        for t in range(z.shape[0]):
            full = np.argsort(-z[t], kind="stable")       # library sort, stable -> id asc on ties
            assert np.array_equal(ids[t], full[:k])
    # k = E returns every id exactly once
    assert all(sorted(r) == list(range(16)) for r in O.topk_ids(z, 16))
    # exact ties go to the lower id, at the boundary and inside the set
    zt = np.array([[1.0, 3.0, 3.0, 2.0, 3.0, 0.0]])
    assert O.topk_ids(zt, 2).tolist() == [[1, 2]]
    assert O.topk_ids(zt, 3).tolist() == [[1, 2, 4]]
    assert O.topk_ids(zt, 4).tolist() == [[1, 2, 4, 3]]


def test_route_weights_and_renorm():
    cfg = SHAPES["tiny"]
    x = _f(gen_hidden(cfg, 16))
    Wg, b = gen_gate(cfg, 0)
    ids, w, p, z = O.gate_route(x, _f(Wg), None, cfg.k, renorm=False)
    assert np.allclose(p.sum(1), 1, atol=1e-12)
    # weights are the softmax entries of the chosen experts, descending
    assert np.array_equal(w, np.take_along_axis(p, ids.astype(np.int64), 1))
    assert (np.diff(w, axis=1) <= 0).all()
    ids2, w2, _, _ = O.gate_route(x, _f(Wg), None, cfg.k, renorm=True)
    assert np.array_equal(ids, ids2)
    assert np.allclose(w2.sum(1), 1, atol=1e-12)
    assert np.allclose(w2 * w.sum(1, keepdims=True), w, rtol=1e-12)
    # a bias large enough decides the route
    bias = np.zeros(cfg.E)
    bias[5] = 100.0
    ids3, _, _, _ = O.gate_route(x, _f(Wg), bias, 1, False)
    assert (ids3 == 5).all()


@pytest.mark.parametrize("name", ["tiny", "qwen", "deepseek", "mixtral"])
def test_prediction_identity_and_monotone_recall(name):
    """Section 4.3: the prediction is the next gate applied to this layer's
    gate input.  If the next layer's input equals this layer's, prediction ==
    the next layer's true routing; and widening the set never loses experts."""
    cfg = SHAPES[name]
    N = 24
    x = _f(gen_hidden(cfg, N))
    Wg1, b1 = gen_gate(cfg, 1)
    b1n = None if b1 is None else b1.numpy()
    true_ids, true_w, p, _ = O.gate_route(x, _f(Wg1), b1n, cfg.k, renorm=False)
    m = default_m(cfg.E, cfg.k)
    pid, pw, pop, _ = O.cross_layer_predict(x, _f(Wg1), b1n, m)
    assert np.array_equal(pid[:, :cfg.k], true_ids)
    assert np.array_equal(pw[:, :cfg.k], true_w)
    assert pop.sum() == N * m
    assert all(len(set(r)) == m for r in pid.tolist())
    # perturbed input: recall of the top-m set is monotone in m and >= top-k accuracy
    x2 = x + 0.3 * np.random.default_rng(3).normal(size=x.shape)
    prev = -1.0
    for mm in range(cfg.k, cfg.E + 1):
        pid2, _, _, _ = O.cross_layer_predict(x2, _f(Wg1), b1n, mm)
        acc_k, rec_m = O.prediction_accuracy(pid2, true_ids, cfg.k)
        assert rec_m >= acc_k - 1e-15 and rec_m >= prev - 1e-15
        prev = rec_m
    assert prev == 1.0          # m = E contains everything


def test_default_m_is_the_75th_percentile_rule():
    # experts strictly above numpy's linearly interpolated 75th percentile of
    # E distinct routing weights
    for E, want in ((60, 15), (64, 16), (8, 2)):
        w = np.random.default_rng(E).permutation(E).astype(np.float64)
        assert int((w > np.percentile(w, 75)).sum()) == want
        assert default_m(E, 1) == want
    assert default_m(8, 4) == 4      # never below k


@pytest.mark.parametrize("N,k,E", [(1, 4, 60), (16, 2, 8), (97, 6, 64), (0, 2, 8)])
def test_permutation_properties(N, k, E):
    rng = np.random.default_rng(N + k)
    ids = np.stack([rng.permutation(E)[:k] for _ in range(N)]).astype(np.int32) if N else np.zeros((0, k), np.int32)
    counts, offsets, perm, inv, order = O.permute(ids, E)
    P = N * k
    flat = ids.reshape(P)
    assert counts.sum() == P and offsets[E] == P and offsets[0] == 0
    assert np.array_equal(np.diff(offsets), counts)
    assert np.array_equal(counts, np.bincount(flat, minlength=E))
    assert sorted(perm.tolist()) == list(range(P))                 # bijection
    assert np.array_equal(perm, np.argsort(flat, kind="stable"))   # library stable sort
    assert np.array_equal(inv[perm], np.arange(P))
    se = flat[perm]
    assert (np.diff(se) >= 0).all()
    for e in range(E):                                             # stability inside an expert
        seg = perm[offsets[e]:offsets[e + 1]]
        assert (np.diff(seg) > 0).all()
    # popularity order: count descending, id ascending
    assert sorted(order.tolist()) == list(range(E))
    keys = [(-counts[e], e) for e in order]
    assert keys == sorted(keys)


def test_near_tie_rows():
    z = np.array([[3.0, 2.0, 1.0, 0.0], [3.0, 2.0, 2.0 - 1e-6, 0.0], [3.0, 3.0 - 1e-7, 1.0, 0.0]])
    assert O.near_tie_rows(z, 2).tolist() == [1, 2]
    assert O.near_tie_rows(z, 1).tolist() == [2]


def test_prediction_accuracy_on_the_papers_near_miss_example():
    """Section 4.2, "Similar Routing Weights": the true top-4 of a token is
    [5, 21, 31, 36], the prediction [5, 11, 21, 36]; three of four are right,
    and the missed expert 31 ranks fifth in the prediction, so a set widened
    to five recovers it."""
    true = np.array([[5, 21, 31, 36]])
    acc_k, rec_m = O.prediction_accuracy(np.array([[5, 11, 21, 36]]), true, 4)
    assert (acc_k, rec_m) == (0.75, 0.75)
    acc_k, rec_m = O.prediction_accuracy(np.array([[5, 11, 21, 36, 31]]), true, 4)
    assert (acc_k, rec_m) == (0.75, 1.0)
    # the denominator is k (not the width of the prediction) and the mean runs over tokens:
    # a second token predicted perfectly, and a third with nothing right
    true3 = np.array([[5, 21, 31, 36], [0, 1, 2, 3], [0, 1, 2, 3]])
    pred3 = np.array([[5, 11, 21, 36, 31, 7], [3, 2, 1, 0, 9, 8], [4, 5, 6, 7, 8, 9]])
    acc_k, rec_m = O.prediction_accuracy(pred3, true3, 4)
    assert acc_k == pytest.approx((0.75 + 1.0 + 0.0) / 3) and rec_m == pytest.approx((1.0 + 1.0 + 0.0) / 3)
    # only the first k true entries count as the true top-k; the arguments are not interchangeable
    assert O.prediction_accuracy(np.array([[9, 8, 5, 21]]), np.array([[5, 21, 9, 8]]), 2) == (0.0, 1.0)
    assert O.prediction_accuracy(np.array([[5, 21, 9, 8]]), np.array([[9, 8, 5, 21]]), 2) == (0.0, 1.0)
    assert O.prediction_accuracy(np.array([[5, 21, 9]]), np.array([[9, 8]]), 2) == (0.0, 0.5)
    assert O.prediction_accuracy(np.array([[9, 8]]), np.array([[5, 21, 9]]), 2) == (0.0, 0.0)


def test_prefill_set_accuracy_hand_case():
    """Prefill metric of section 4.2 / table 1 (set level): the share of the experts
    a layer really activates, over all tokens, that the prediction's union holds."""
    true = np.array([[1, 2], [2, 3], [3, 4]])            # union {1,2,3,4}
    pred = np.array([[1, 2, 9], [2, 9, 8], [3, 9, 7]])   # union {1,2,3,7,8,9}: 3 of the 4 true ones
    assert O.prefill_set_accuracy(pred, true) == 0.75
    # not symmetric: 3 of the 6 predicted are true
    assert O.prefill_set_accuracy(true, pred) == 0.5
    assert O.prefill_set_accuracy(true, true) == 1.0
    assert O.prefill_set_accuracy(np.array([[5, 6]]), true) == 0.0
