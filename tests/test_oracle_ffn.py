"""Pins of the dequantisation and FFN oracle: exact round trips, a group worked
by hand, error bounds, and the one-expert case against a dense SwiGLU MLP
computed with torch's own fp64 silu and matmul."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import moe as O
from workloads import SHAPES, gen_hidden, gen_gate, gen_expert, gen_shared_gate, quantize_sym


def _f(t):
    return t.to(torch.float32).numpy()


def test_dequant_hand_worked_group():
    # one row, two groups of 4, int4.  Group 0: max|w| = 0.7 -> s = fp16(0.1);
    # group 1 all zero -> s = 1, q = 0.
    w = np.array([[0.7, -0.35, 0.04, -0.7, 0.0, 0.0, 0.0, 0.0]])
    q, s = O.quantize_sym(w, 4, 4)
    s0 = np.float16(0.7 / 7)
    assert s.dtype == np.float16 and s[0, 0] == s0 and s[0, 1] == np.float16(1.0)
    # -0.35 / fp16(0.1): fp16(0.1) = 0.0999755859375 -> -3.5009 -> -4 ; 0.04/s = 0.4001 -> 0
    assert q.tolist() == [[7, -4, 0, -7, 0, 0, 0, 0]]
    packed = O.pack_codes(q, 4)
    # nibble u = q + 8, low nibble is the even column: (15 | 4<<4), (8 | 1<<4), 0x88, 0x88
    assert packed.tolist() == [[0x4F, 0x18, 0x88, 0x88]]
    assert np.array_equal(O.unpack_codes(packed, 4), q)
    d = O.dequant(packed, s, 4, 4)
    assert d[0, 0] == 7 * float(s0) and d[0, 1] == -4 * float(s0) and d[0, 4] == 0.0
    # int8 two's complement storage
    q8 = np.array([[-127, -1, 0, 127]])
    p8 = O.pack_codes(q8, 8)
    assert p8.tolist() == [[0x81, 0xFF, 0x00, 0x7F]]
    assert np.array_equal(O.unpack_codes(p8, 8), q8)


@pytest.mark.parametrize("bits,group", [(8, 64), (4, 128)])
def test_quant_round_trip_and_error_bound(bits, group):
    rng = np.random.default_rng(bits)
    w = rng.normal(size=(48, 4 * group)) * 0.02
    w[3, :group] = 0.0                                  # an all-zero group
    q, s = O.quantize_sym(w, bits, group)
    qmax = 127 if bits == 8 else 7
    assert np.abs(q).max() <= qmax
    d = O.dequant(O.pack_codes(q, bits), s, bits, group)
    sfull = np.repeat(s.astype(np.float64), group, axis=1)
    assert (np.abs(w - d) <= sfull / 2 + 1e-18).all()
    # q*s is exact in fp32 as well as in fp64
    d32 = (q.astype(np.float32) * np.repeat(s.astype(np.float32), group, axis=1)).astype(np.float64)
    assert np.array_equal(d, d32)
    # re-quantising the dequantised weights with the same scales gives the same codes
    q2 = np.clip(np.rint(d / sfull), -qmax, qmax).astype(np.int32)
    assert np.array_equal(q2, q)
    # every non-zero group uses its full range
    gmax = np.abs(q).reshape(48, 4, group).max(axis=-1)
    assert (gmax[np.abs(w).reshape(48, 4, group).max(-1) > 0] == qmax).all()
    assert s[3, 0] == np.float16(1.0) and (q[3, :group] == 0).all()


@pytest.mark.parametrize("bits,group", [(8, 64), (4, 128), (2, 128)])
def test_workload_quantizer_agrees_with_oracle_reading(bits, group):
    """The generator's stored weights obey the oracle's format: same scales,
    and codes that differ at most where w/s sits on a rounding boundary."""
    g = torch.Generator().manual_seed(5)
    w = torch.randn(32, 2 * group, generator=g) * 0.02
    codes, s = quantize_sym(w, bits, group)
    q_ref, s_ref = O.quantize_sym(w.numpy().astype(np.float64), bits, group)
    assert np.array_equal(s.numpy(), s_ref)
    q = O.unpack_codes(codes.numpy(), bits)
    assert np.abs(q - q_ref).max() <= (2 if bits == 2 else 1) and (q != q_ref).mean() < 1e-3


def _dense_swiglu_torch(x, W1, W3, W2):
    x, W1, W3, W2 = (torch.from_numpy(np.ascontiguousarray(a)).double() for a in (x, W1, W3, W2))
    return ((F.silu(x @ W1.T) * (x @ W3.T)) @ W2.T).numpy()


def _oracle_expert(ex):
    ex = ex.cpu()
    return O.OracleExpert(ex.w1.numpy(), ex.s1.numpy(), ex.w3.numpy(), ex.s3.numpy(),
                          ex.w2.numpy(), ex.s2.numpy(), ex.bits, ex.group)


def test_silu_matches_torch():
    a = np.linspace(-30, 30, 1001)
    assert np.allclose(O.silu(a), F.silu(torch.from_numpy(a)).numpy(), rtol=1e-14, atol=1e-300)


def test_ffn_one_expert_is_a_dense_swiglu_mlp():
    cfg = SHAPES["tiny"]
    x = _f(gen_hidden(cfg, 5))
    ex = _oracle_expert(gen_expert(cfg, 0, 3))
    assert ex.W1.shape == (cfg.I, cfg.H) and ex.W2.shape == (cfg.H, cfg.I)
    ids = np.full((5, 1), 3, dtype=np.int32)
    w = np.ones((5, 1))
    y = O.moe_ffn(x, ids, w, {3: ex})
    ref = _dense_swiglu_torch(x.astype(np.float64), ex.W1, ex.W3, ex.W2)
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-15)
    # swapping gate and up projections, or dropping silu, must not pass
    wrong = _dense_swiglu_torch(x.astype(np.float64), ex.W3, ex.W1, ex.W2)
    assert not np.allclose(y, wrong, rtol=1e-3)


def test_ffn_combination_linearity_and_shared_term():
    cfg = SHAPES["tiny"]
    N = 6
    x = _f(gen_hidden(cfg, N))
    Wg, _ = gen_gate(cfg, 0)
    ids, w, _, _ = O.gate_route(x, _f(Wg), None, cfg.k, True)
    experts = {e: _oracle_expert(gen_expert(cfg, 0, e)) for e in range(cfg.E)}
    y = O.moe_ffn(x, ids, w, experts)
    # definition by pairs with torch's dense MLP per expert
    ref = np.zeros_like(y)
    for t in range(N):
        for j in range(cfg.k):
            ex = experts[int(ids[t, j])]
            ref[t] += w[t, j] * _dense_swiglu_torch(x[t:t + 1].astype(np.float64), ex.W1, ex.W3, ex.W2)[0]
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-15)
    # linear in the routing weights
    y2 = O.moe_ffn(x, ids, 2.5 * w, experts)
    assert np.allclose(y2, 2.5 * y, rtol=1e-12)
    wa = w.copy(); wa[:, 1] = 0
    wb = w.copy(); wb[:, 0] = 0
    assert np.allclose(O.moe_ffn(x, ids, wa, experts) + O.moe_ffn(x, ids, wb, experts), y, rtol=1e-12, atol=1e-15)
    # shared experts: ungated term alone, then the sigmoid gate
    sh = [_oracle_expert(gen_expert(cfg, 0, 0, shared=False)), _oracle_expert(gen_expert(cfg, 0, 1))]
    y_sh = O.moe_ffn(x, ids, np.zeros_like(w), experts, shared=sh)
    ref_sh = sum(_dense_swiglu_torch(x.astype(np.float64), s.W1, s.W3, s.W2) for s in sh)
    assert np.allclose(y_sh, ref_sh, rtol=1e-12, atol=1e-15)
    sg = np.random.default_rng(0).normal(size=cfg.H) / 16
    y_g = O.moe_ffn(x, ids, np.zeros_like(w), experts, shared=sh, shared_gate=sg)
    gate = torch.sigmoid(torch.from_numpy(x.astype(np.float64) @ sg)).numpy()
    assert np.allclose(y_g, gate[:, None] * ref_sh, rtol=1e-12, atol=1e-15)
    # routed + shared add
    y_all = O.moe_ffn(x, ids, w, experts, shared=sh, shared_gate=sg)
    assert np.allclose(y_all, y + y_g, rtol=1e-12, atol=1e-15)


def test_ffn_rows_subset():
    cfg = SHAPES["tiny"]
    x = _f(gen_hidden(cfg, 8))
    Wg, _ = gen_gate(cfg, 0)
    ids, w, _, _ = O.gate_route(x, _f(Wg), None, cfg.k, True)
    experts = {e: _oracle_expert(gen_expert(cfg, 0, e)) for e in range(cfg.E)}
    y = O.moe_ffn(x, ids, w, experts)
    assert np.array_equal(O.moe_ffn_rows(x, ids, w, experts, rows=[5, 2]), y[[5, 2]])


def _grouped_vs_pairs(name, N, layer=0):
    cfg = SHAPES[name]
    x = _f(gen_hidden(cfg, N))
    Wg, b = gen_gate(cfg, layer)
    ids, w, _, _ = O.gate_route(x, _f(Wg), None if b is None else b.numpy(), cfg.k, cfg.renorm)
    experts = {e: _oracle_expert(gen_expert(cfg, layer, e)) for e in sorted(set(ids.ravel().tolist()))}
    shared = [_oracle_expert(gen_expert(cfg, layer, s, shared=True)) for s in range(cfg.n_shared)]
    sg = gen_shared_gate(cfg, layer)
    sg = None if sg is None else _f(sg)
    y_pairs = O.moe_ffn(x, ids, w, experts, shared, sg)
    y_grouped = O.moe_ffn_grouped(x, ids, w, experts, shared, sg)
    return y_pairs, y_grouped, ids


def test_grouped_ffn_form_equals_the_pairwise_definition_tiny():
    y_pairs, y_grouped, ids = _grouped_vs_pairs("tiny", 16)
    assert len(set(ids.ravel().tolist())) > 2
    assert np.allclose(y_grouped, y_pairs, rtol=1e-12, atol=1e-16)
    # a dropped routing weight or a scatter to the wrong token would not pass
    assert not np.allclose(y_grouped[::-1], y_pairs, rtol=1e-3)


def test_grouped_ffn_form_equals_the_pairwise_definition_qwen_rows():
    """Eight token rows of the Qwen1.5-MoE-shaped layer (60 experts top-4, gated shared expert)."""
    y_pairs, y_grouped, ids = _grouped_vs_pairs("qwen", 8)
    assert np.allclose(y_grouped, y_pairs, rtol=1e-12, atol=1e-16)


def test_grouped_ffn_repeated_expert_and_empty_cases():
    cfg = SHAPES["tiny"]
    x = _f(gen_hidden(cfg, 4))
    experts = {e: _oracle_expert(gen_expert(cfg, 0, e)) for e in (1, 2)}
    ids = np.array([[1, 2], [2, 1], [1, 2], [2, 1]], dtype=np.int32)
    w = np.random.default_rng(1).uniform(0.1, 1.0, size=(4, 2))
    assert np.allclose(O.moe_ffn_grouped(x, ids, w, experts), O.moe_ffn(x, ids, w, experts), rtol=1e-12, atol=1e-16)
    empty = O.moe_ffn_grouped(x[:0], ids[:0], w[:0], experts)
    assert empty.shape == (0, cfg.H)


def test_int2_format_hand_worked_group():
    """The low-precision copy of section 4.5, one row, two groups of 4.  Group 0: max|w| = 0.6 ->
    s = fp16(0.2); levels -0.6, -0.2, 0.2, 0.6 (times the rounded s).  Group 1 is all zero -> s = 0."""
    w = np.array([[0.6, -0.35, 0.05, -0.6, 0.0, 0.0, 0.0, 0.0]])
    q, s = O.quantize_sym(w, 2, 4)
    s0 = np.float16(0.6 / 3)
    assert s.dtype == np.float16 and s[0, 0] == s0 and s[0, 1] == np.float16(0.0)
    # 0.6 -> +3 ; -0.35 / 0.2 = -1.75 -> nearest odd level -1 (field (-1.75 + 3) / 2 = 0.625 -> 1);
    # 0.05 -> +1 ; -0.6 -> -3 ; the zero group takes field 0 = level -3 times a zero scale
    assert q.tolist() == [[3, -1, 1, -3, -3, -3, -3, -3]]
    packed = O.pack_codes(q, 2)
    # fields u = (q + 3) / 2 = 3, 1, 2, 0 -> byte 3 | 1 << 2 | 2 << 4 | 0 << 6 = 0x27 ; second byte 0
    assert packed.tolist() == [[0x27, 0x00]]
    assert np.array_equal(O.unpack_codes(packed, 2), q)
    d = O.dequant(packed, s, 2, 4)
    assert d[0, 0] == 3 * float(s0) and d[0, 1] == -float(s0) and d[0, 3] == -3 * float(s0)
    assert (d[0, 4:] == 0).all()


def test_int2_round_trip_and_error_bound():
    rng = np.random.default_rng(2)
    group = 128
    w = rng.normal(size=(40, 4 * group)) * 0.02
    w[5, group:2 * group] = 0.0
    q, s = O.quantize_sym(w, 2, group)
    assert set(np.unique(q).tolist()) <= {-3, -1, 1, 3}
    packed = O.pack_codes(q, 2)
    assert packed.shape == (40, 4 * group // 4) and np.array_equal(O.unpack_codes(packed, 2), q)
    d = O.dequant(packed, s, 2, group)
    sfull = np.repeat(s.astype(np.float64), group, axis=1)
    # nearest of the levels -3s .. 3s: off by at most s, plus what rounding s to fp16 moves the outermost level
    assert (np.abs(w - d) <= sfull * (1 + 3 * 2.0 ** -11) + 1e-18).all()
    # q*s is exact in fp32; re-quantising the dequantised weights with the same scales gives the same codes
    d32 = (q.astype(np.float32) * np.repeat(s.astype(np.float32), group, axis=1)).astype(np.float64)
    assert np.array_equal(d, d32)
    with np.errstate(divide="ignore", invalid="ignore"):
        u2 = np.where(sfull > 0, np.rint((d / sfull + 3) / 2), 0)
    assert np.array_equal(2 * np.clip(u2, 0, 3).astype(np.int32) - 3, q)
    # every non-zero group reaches an outermost level; the all-zero group dequantises to zero
    gmax = np.abs(q).reshape(40, 4, group).max(axis=-1)
    assert (gmax[np.abs(w).reshape(40, 4, group).max(-1) > 0] == 3).all()
    assert s[5, 1] == 0 and (d[5, group:2 * group] == 0).all()
    # coarser than the 4-bit format on the same weights, finer than nothing: error ordering
    q4, s4 = O.quantize_sym(w, 4, group)
    d4 = O.dequant(O.pack_codes(q4, 4), s4, 4, group)
    assert np.abs(w - d4).mean() < np.abs(w - d).mean() < np.abs(w).mean()


def test_zero_point_format_hand_worked_group():
    """The asymmetric format of the paper's quantiser (HQQ, section 4.5): one row, one group of 4, int4.
    min = -0.1, max = 0.5 -> s = fp16(0.6 / 15) = fp16(0.04), z = fp16(0.1 / s)."""
    w = np.array([[-0.1, 0.5, 0.0, 0.21]])
    u, s, z = O.quantize_asym(w, 4, 4)
    s0 = np.float16(0.6 / 15)
    z0 = np.float16(0.1 / float(s0))
    assert s[0, 0] == s0 and z[0, 0] == z0 and 2.4 < float(z0) < 2.6
    # fields: -0.1 / s + z = 0 ; 0.5 / s + z = 15.0 ; 0 -> z = 2.5 (ties to even: 2) ; 0.21 / 0.04 + 2.5 = 7.75 -> 8
    assert u.tolist() == [[0, 15, round(float(z0)), 8]]
    packed = O.pack_fields(u, 4)
    assert packed.tolist() == [[0xF0, 0x80 | round(float(z0))]]
    assert np.array_equal(O.unpack_fields(packed, 4), u)
    d = O.dequant_zp(packed, s, z, 4, 4)
    assert d[0, 1] == (15 - float(z0)) * float(s0) and d[0, 0] == (0 - float(z0)) * float(s0)
    # the symmetric formats are the special case z = 8 (int4) / 128 (int8, offset binary) / 1.5 with twice the scale (int2)
    rng = np.random.default_rng(0)
    w2 = rng.normal(size=(4, 256)) * 0.02
    for bits, zsym, smul in ((4, 8.0, 1.0), (8, 128.0, 1.0), (2, 1.5, 2.0)):
        q, ss = O.quantize_sym(w2, bits, 128)
        ufield = O.unpack_fields(O.pack_codes(q, bits) if bits != 8 else (q + 128).astype(np.uint8), bits)
        dz = O.dequant_zp(O.pack_fields(ufield, bits), (ss.astype(np.float64) * smul).astype(np.float16),
                          np.full(ss.shape, zsym, np.float16), bits, 128)
        assert np.array_equal(dz, O.dequant(O.pack_codes(q, bits), ss, bits, 128))


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_zero_point_quantiser_error_bounds_and_refinement(bits):
    rng = np.random.default_rng(bits)
    group = 128
    w = rng.normal(size=(24, 3 * group)) * 0.02 + 0.01          # off-centre: where a zero-point pays
    w[2, :group] = 0.37                                         # a constant group
    u, s, z = O.quantize_asym(w, bits, group)
    qmax = (1 << bits) - 1
    assert u.min() >= 0 and u.max() <= qmax
    d = O.dequant_zp(O.pack_fields(u, bits), s, z, bits, group)
    sfull = np.repeat(s.astype(np.float64), group, axis=1)
    # nearest level of a grid that covers [min, max] up to the fp16 rounding of s and z
    assert (np.abs(w - d) <= sfull * (0.5 + qmax * 2.0 ** -10) + 1e-12).all()
    assert s[2, 0] == np.float16(1.0) and np.abs(d[2, :group] - 0.37).max() <= 0.5
    # asymmetric beats symmetric on off-centre weights at the same width
    q, ss = O.quantize_sym(w, bits, group)
    dsym = O.dequant(O.pack_codes(q, bits), ss, bits, group)
    assert np.abs(w - d)[3:].mean() < np.abs(w - dsym)[3:].mean()
    # the half-quadratic refinement of the zero-point never loses against its starting point (it keeps the best)
    u2, s2, z2 = O.quantize_asym(w, bits, group, hqq_iters=20)
    d2 = O.dequant_zp(O.pack_fields(u2, bits), s2, z2, bits, group)
    assert np.array_equal(s2, s)
    e1 = np.abs(w - d).reshape(24, 3, group).mean(-1)
    e2 = np.abs(w - d2).reshape(24, 3, group).mean(-1)
    assert (e2 <= e1 * 1.02 + 1e-9).all() and e2.mean() <= e1.mean()


def test_shrinkage_operator_of_the_half_quadratic_solver():
    x = np.array([-2.0, -0.01, 0.0, 0.01, 0.5, 3.0])
    y = O._shrink_lp(x, beta=10.0, p=0.7)
    # |x| - |x|^(p-1)/beta, clipped at zero, sign kept: small entries vanish, large ones barely move
    assert y[2] == 0 and y[1] == 0 and y[3] == 0
    assert np.isclose(y[5], 3.0 - 3.0 ** (-0.3) / 10) and np.isclose(y[0], -(2.0 - 2.0 ** (-0.3) / 10))
    assert np.isclose(y[4], 0.5 - 0.5 ** (-0.3) / 10)
    # p = 1 is the ordinary soft threshold
    assert np.allclose(O._shrink_lp(x, 4.0, 1.0), np.sign(x) * np.maximum(np.abs(x) - 0.25, 0))
