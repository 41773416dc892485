"""CPU oracle for the per-layer MoE forward of Fate's offloaded inference.

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 numpy; shares no code with the
HIP library and is imported only by tests, the smoke check and the
cpu_baseline leg of the benchmark.  Every function is the plain definition of
what the hot path computes, acting on the exact values of the stored inputs
(bf16 / fp16 / integer codes widened to fp64).

Paper basis: the gate is a softmax over all experts whose routing weights sum
to 1, and the k largest are selected (section 2.1; section 4.2 "Similar
Routing Weights").  The cross-layer prediction feeds block i's gate input to
block i+1's gate (section 4.3), optionally widened beyond k (section 4.2,
75th-percentile rule), and in prefill is aggregated into a per-expert
popularity count (section 4.3 "Prefill Stage").  Experts are stored
quantised and dequantised before compute (section 4.1 steps 5-6; section
4.5).  The SwiGLU expert body and the shared / fine-grained structure are the
standard ones of section 2.1.

Pins (tests/test_oracle_*.py): softmax against scipy and its invariants,
top-k against a full sort and constructed ties, prediction identity,
permutation against numpy's stable argsort and bijection properties,
dequantisation round trips and a hand-computed group, FFN against a torch
fp64 dense SwiGLU MLP in the one-expert case plus linearity properties,
the expert-by-expert form of the FFN against the pair-by-pair definition,
the accuracy metrics against the paper's near-miss example and hand cases.
"""
import numpy as np

# ----------------------------------------------------------------------------
# routing
# ----------------------------------------------------------------------------


def gate_logits(x, Wg, bias=None):
    """z[t,e] = sum_h x[t,h] * Wg[e,h] + bias[e], in fp64."""
    x = np.asarray(x, dtype=np.float64)
    Wg = np.asarray(Wg, dtype=np.float64)
    z = x @ Wg.T
    if bias is not None:
        z = z + np.asarray(bias, dtype=np.float64)[None, :]
    return z


def softmax(z):
    """Routing weights over all experts; each row sums to 1."""
    z = np.asarray(z, dtype=np.float64)
    zs = z - z.max(axis=-1, keepdims=True)
    ez = np.exp(zs)
    return ez / ez.sum(axis=-1, keepdims=True)


def topk_ids(z, k):
    """The k experts with the highest logits; ties go to the lower id.
    Output order: logit descending, then id ascending."""
    z = np.asarray(z, dtype=np.float64)
    N, E = z.shape
    assert 1 <= k <= E
    ids = np.empty((N, k), dtype=np.int32)
    for t in range(N):
        order = sorted(range(E), key=lambda e: (-z[t, e], e))
        ids[t] = order[:k]
    return ids


def gate_route(x, Wg, bias, k, renorm):
    """Gate of one layer.  Returns (ids [N,k] i32, w [N,k] f64, probs [N,E] f64, z)."""
    z = gate_logits(x, Wg, bias)
    p = softmax(z)
    ids = topk_ids(z, k)
    w = np.take_along_axis(p, ids.astype(np.int64), axis=1)
    if renorm:
        w = w / w.sum(axis=1, keepdims=True)
    return ids, w, p, z


def cross_layer_predict(x_l, Wg_next, bias_next, m):
    """Prediction of layer l+1's routing from layer l's gate input: the next
    layer's gate applied to x_l, top-m (m >= k widens the prefetch set).
    pred_pop[e] = number of tokens whose top-m contains e."""
    z = gate_logits(x_l, Wg_next, bias_next)
    p = softmax(z)
    ids = topk_ids(z, m)
    w = np.take_along_axis(p, ids.astype(np.int64), axis=1)
    E = z.shape[1]
    pop = np.zeros(E, dtype=np.int32)
    for t in range(ids.shape[0]):
        for j in range(m):
            pop[ids[t, j]] += 1
    return ids, w, pop, z


def near_tie_rows(z, k, margin=1e-5):
    """Rows whose sorted logits have a gap below `margin` between ranks j and
    j+1 for some j <= k (1-based); such rows may legitimately differ between
    fp32 and fp64 routing and are reported apart."""
    z = np.asarray(z, dtype=np.float64)
    zs = -np.sort(-z, axis=1)
    kk = min(k, z.shape[1] - 1)
    gaps = zs[:, :kk] - zs[:, 1:kk + 1]
    return np.nonzero((gaps < margin).any(axis=1))[0]


# ----------------------------------------------------------------------------
# permutation
# ----------------------------------------------------------------------------


def permute(ids, E):
    """Token-to-expert grouping.  Pair index p = t*k + j.

    counts[e]  = number of pairs routed to e
    offsets    = exclusive prefix sum of counts, offsets[E] = N*k
    perm[s]    = pair index at sorted position s, ordered by (expert, pair)
    inv_perm   = inverse of perm
    expert_order = experts by (count descending, id ascending)
    """
    ids = np.asarray(ids)
    N, k = ids.shape
    P = N * k
    flat = ids.reshape(P)
    counts = np.zeros(E, dtype=np.int32)
    for p in range(P):
        counts[flat[p]] += 1
    offsets = np.zeros(E + 1, dtype=np.int32)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    cursor = offsets[:E].copy()
    perm = np.empty(P, dtype=np.int32)
    inv = np.empty(P, dtype=np.int32)
    for p in range(P):
        e = flat[p]
        perm[cursor[e]] = p
        inv[p] = cursor[e]
        cursor[e] += 1
    order = np.array(sorted(range(E), key=lambda e: (-int(counts[e]), e)), dtype=np.int32)
    return counts, offsets, perm, inv, order


# ----------------------------------------------------------------------------
# quantised weights
# ----------------------------------------------------------------------------


def unpack_codes(codes_u8, bits):
    """Canonical stored codes -> signed integer codes [rows, K] (int32).
    int8: two's complement bytes.  int4: nibble u = q + 8, low nibble first.
    int2: field u in 0..3, four per byte, column 4b+i in bits 2i..2i+1 of byte b; the signed code
    is the odd integer q = 2u - 3 (levels -3, -1, 1, 3 times the group's scale)."""
    c = np.asarray(codes_u8, dtype=np.uint8)
    if bits == 8:
        return c.view(np.int8).astype(np.int32)
    if bits == 2:
        rows, quarter = c.shape
        q = np.empty((rows, quarter * 4), dtype=np.int32)
        for i in range(4):
            q[:, i::4] = 2 * ((c >> (2 * i)) & 0x3).astype(np.int32) - 3
        return q
    assert bits == 4
    rows, half = c.shape
    q = np.empty((rows, half * 2), dtype=np.int32)
    q[:, 0::2] = (c & 0x0F).astype(np.int32) - 8
    q[:, 1::2] = (c >> 4).astype(np.int32) - 8
    return q


def dequant(codes_u8, scales_f16, bits, group):
    """w[r, c] = q[r, c] * s[r, c // group] in fp64 (symmetric: zero-point 0; for the 2-bit
    format q runs over the odd integers -3 .. 3)."""
    q = unpack_codes(codes_u8, bits).astype(np.float64)
    s = np.asarray(scales_f16, dtype=np.float16).astype(np.float64)
    rows, K = q.shape
    assert s.shape == (rows, K // group)
    return q * np.repeat(s, group, axis=1)


def quantize_sym(w, bits, group):
    """Reference symmetric group quantiser: s = fp16(max|w|/qmax) per group
    (1 for an all-zero group), q = round-half-even(w/s) clamped to +-qmax with
    the rounded s.  Returns (signed codes int32 [rows,K], scales fp16).

    bits = 2 (the low-precision copy of section 4.5): a symmetric code with a zero level would
    use three of the four codes, so the four levels are the odd multiples -3, -1, 1, 3 of the
    scale s = fp16(max|w|/3) (s = 0 for an all-zero group, which then dequantises to zero);
    q is the nearest level, computed with the rounded s, ties to the field value that is even."""
    w = np.asarray(w, dtype=np.float64)
    rows, K = w.shape
    if bits == 2:
        wg = w.reshape(rows, K // group, group)
        s = (np.abs(wg).max(axis=-1) / 3).astype(np.float16)
        sd = s.astype(np.float64)[..., None]
        with np.errstate(divide="ignore", invalid="ignore"):
            u = np.where(sd > 0, np.rint((wg / sd + 3) / 2), 0)
        u = np.clip(u, 0, 3).astype(np.int32)
        return (2 * u - 3).reshape(rows, K), s
    qmax = 127 if bits == 8 else 7
    wg = w.reshape(rows, K // group, group)
    s = (np.abs(wg).max(axis=-1) / qmax).astype(np.float16)
    s = np.where(s == 0, np.float16(1.0), s)
    q = np.clip(np.rint(wg / s.astype(np.float64)[..., None]), -qmax, qmax).astype(np.int32)
    return q.reshape(rows, K), s


def pack_codes(q, bits):
    """Signed codes -> canonical stored bytes (inverse of unpack_codes)."""
    q = np.asarray(q, dtype=np.int32)
    if bits == 8:
        return q.astype(np.int8).view(np.uint8)
    if bits == 2:
        u = ((q + 3) // 2).astype(np.uint8)
        return (u[:, 0::4] | (u[:, 1::4] << 2) | (u[:, 2::4] << 4) | (u[:, 3::4] << 6)).astype(np.uint8)
    u = (q + 8).astype(np.uint8)
    return (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)


# -- asymmetric (zero-point) group format: what HQQ, the quantiser the paper uses (section 4.5), produces --


def unpack_fields(codes_u8, bits):
    """Canonical stored bytes -> the unsigned fields u in [0, 2^bits) [rows, K] (int32): the nibble
    (int4), the 2-bit field (int2) or the byte (int8) as stored by the asymmetric quantiser."""
    c = np.asarray(codes_u8, dtype=np.uint8)
    if bits == 8:
        return c.astype(np.int32)
    per = 8 // bits
    rows, nb = c.shape
    u = np.empty((rows, nb * per), dtype=np.int32)
    for i in range(per):
        u[:, i::per] = (c >> (bits * i)) & ((1 << bits) - 1)
    return u


def pack_fields(u, bits):
    """Inverse of unpack_fields."""
    u = np.asarray(u, dtype=np.int32)
    if bits == 8:
        return u.astype(np.uint8)
    per = 8 // bits
    out = np.zeros((u.shape[0], u.shape[1] // per), dtype=np.uint8)
    for i in range(per):
        out |= (u[:, i::per] << (bits * i)).astype(np.uint8)
    return out


def dequant_zp(codes_u8, scales_f16, zeros_f16, bits, group):
    """w[r, c] = (u[r, c] - z[r, c // group]) * s[r, c // group] in fp64, u the stored unsigned field,
    s and z one fp16 value per group."""
    u = unpack_fields(codes_u8, bits).astype(np.float64)
    s = np.repeat(np.asarray(scales_f16, dtype=np.float16).astype(np.float64), group, axis=1)
    z = np.repeat(np.asarray(zeros_f16, dtype=np.float16).astype(np.float64), group, axis=1)
    assert s.shape == u.shape == z.shape
    return (u - z) * s


def _shrink_lp(x, beta, p):
    """Generalised soft threshold of the half-quadratic solver: sign(x) * max(|x| - |x|^(p-1) / beta, 0)."""
    ax = np.abs(x)
    with np.errstate(divide="ignore"):
        t = np.where(ax > 0, ax ** (p - 1.0) / beta, 0.0)
    return np.sign(x) * np.maximum(ax - t, 0.0)


def quantize_asym(w, bits, group, hqq_iters=0, p=0.7, beta=10.0, kappa=1.01):
    """Asymmetric group quantiser: per group s = fp16((max - min) / (2^bits - 1)) (1 for a constant
    group) and zero-point z = fp16(-min / s), u = clamp(round-half-even(w / s + z), 0, 2^bits - 1).
    hqq_iters > 0 refines the zero-point the way Half-Quadratic Quantization (Badri & Shaji, 2023)
    does, with the scale kept fixed: alternate the l_p shrinkage of the residual with the closed-form
    zero-point z = mean(u - (w - e) / s), beta growing by kappa per step; the best zero-point seen (mean
    |residual|) is kept.  Returns (fields int32 [rows, K], scales fp16, zeros fp16)."""
    w = np.asarray(w, dtype=np.float64)
    rows, K = w.shape
    qmax = (1 << bits) - 1
    wg = w.reshape(rows, K // group, group)
    lo, hi = wg.min(axis=-1), wg.max(axis=-1)
    s = ((hi - lo) / qmax).astype(np.float16)
    s = np.where(s == 0, np.float16(1.0), s)
    sd = s.astype(np.float64)[..., None]
    z = (-lo[..., None] / sd)

    def fields(zz):
        return np.clip(np.rint(wg / sd + zz), 0, qmax)

    if hqq_iters > 0:
        best_z, best_err = z.copy(), np.abs(wg - (fields(z) - z) * sd).mean(axis=-1, keepdims=True)
        b = beta
        for _ in range(hqq_iters):
            u = fields(z)
            e = _shrink_lp(wg - (u - z) * sd, b, p)
            z = (u - (wg - e) / sd).mean(axis=-1, keepdims=True)
            b *= kappa
            err = np.abs(wg - (fields(z) - z) * sd).mean(axis=-1, keepdims=True)
            better = err < best_err
            best_z = np.where(better, z, best_z)
            best_err = np.where(better, err, best_err)
        z = best_z
    z16 = z[..., 0].astype(np.float16)
    u = np.clip(np.rint(wg / sd + z16.astype(np.float64)[..., None]), 0, qmax).astype(np.int32)
    return u.reshape(rows, K), s, z16


class OracleExpert:
    """Dequantised fp64 matrices of one SwiGLU expert (zero-points z1, z3, z2 given: the asymmetric format)."""

    def __init__(self, w1, s1, w3, s3, w2, s2, bits, group, z1=None, z3=None, z2=None):
        if z1 is not None:
            self.W1 = dequant_zp(w1, s1, z1, bits, group)
            self.W3 = dequant_zp(w3, s3, z3, bits, group)
            self.W2 = dequant_zp(w2, s2, z2, bits, group)
            return
        self.W1 = dequant(w1, s1, bits, group)   # [I, H]
        self.W3 = dequant(w3, s3, bits, group)   # [I, H]
        self.W2 = dequant(w2, s2, bits, group)   # [H, I]


# ----------------------------------------------------------------------------
# expert FFN
# ----------------------------------------------------------------------------


def silu(a):
    a = np.asarray(a, dtype=np.float64)
    return a / (1.0 + np.exp(-a))


def expert_ffn(x_rows, ex):
    """SwiGLU expert on rows of x: W2 (silu(W1 x) * (W3 x)).  Also returns h."""
    x_rows = np.asarray(x_rows, dtype=np.float64)
    h = silu(x_rows @ ex.W1.T) * (x_rows @ ex.W3.T)
    return h @ ex.W2.T, h


def moe_ffn(x, ids, w, experts, shared=(), shared_gate=None):
    """y[t] = sum_j w[t,j] * FFN_{ids[t,j]}(x[t]) + sum_s gate_s(t) * FFN_s(x[t]).

    experts: mapping e -> OracleExpert (only routed-to experts are needed).
    shared: sequence of OracleExpert, always active; gate_s = 1, or
    sigmoid(x[t] . shared_gate) when a gate vector is given.
    """
    x = np.asarray(x, dtype=np.float64)
    N, H = x.shape
    y = np.zeros((N, H), dtype=np.float64)
    ids = np.asarray(ids)
    w = np.asarray(w, dtype=np.float64)
    for t in range(N):
        for j in range(ids.shape[1]):
            out, _ = expert_ffn(x[t:t + 1], experts[int(ids[t, j])])
            y[t] += w[t, j] * out[0]
    if len(shared):
        if shared_gate is not None:
            sg = np.asarray(shared_gate, dtype=np.float64)
            g = 1.0 / (1.0 + np.exp(-(x @ sg)))
        else:
            g = np.ones(N, dtype=np.float64)
        for ex in shared:
            out, _ = expert_ffn(x, ex)
            y += g[:, None] * out
    return y


def moe_ffn_grouped(x, ids, w, experts, shared=(), shared_gate=None):
    """The same sum as moe_ffn, taken expert by expert instead of token by token:
    the rows routed to an expert go through it as one fp64 matrix product, and
    their outputs are scattered back with their routing weights.  Nothing else
    changes (same dequantised matrices, same SwiGLU body), so it agrees with
    moe_ffn up to the order of the fp64 additions; it exists because the
    pair-by-pair form takes minutes on a full prefill layer.  Pinned against
    moe_ffn in tests/test_oracle_ffn.py."""
    x = np.asarray(x, dtype=np.float64)
    N, H = x.shape
    ids = np.asarray(ids)
    w = np.asarray(w, dtype=np.float64)
    y = np.zeros((N, H), dtype=np.float64)
    for e in sorted(set(int(v) for v in ids.ravel())):
        t_idx, j_idx = np.nonzero(ids == e)
        out, _ = expert_ffn(x[t_idx], experts[e])
        np.add.at(y, t_idx, w[t_idx, j_idx][:, None] * out)
    if len(shared):
        if shared_gate is not None:
            g = 1.0 / (1.0 + np.exp(-(x @ np.asarray(shared_gate, dtype=np.float64))))
        else:
            g = np.ones(N, dtype=np.float64)
        for ex in shared:
            out, _ = expert_ffn(x, ex)
            y += g[:, None] * out
    return y


def moe_ffn_rows(x, ids, w, experts, shared=(), shared_gate=None, rows=None):
    """moe_ffn restricted to the token rows in `rows` (for sampled parity)."""
    rows = list(range(np.asarray(x).shape[0])) if rows is None else list(rows)
    xs = np.asarray(x, dtype=np.float64)[rows]
    return moe_ffn(xs, np.asarray(ids)[rows], np.asarray(w)[rows], experts, shared, shared_gate)


# ----------------------------------------------------------------------------
# accuracy metrics of the prediction (reported, not graded against the paper)
# ----------------------------------------------------------------------------


def prediction_accuracy(pred_ids, true_ids, k):
    """Decode metric: mean over tokens of |pred_top-k ∩ true_top-k| / k, and
    the recall of the widened set |pred_top-m ∩ true_top-k| / k."""
    pred_ids = np.asarray(pred_ids)
    true_ids = np.asarray(true_ids)
    N = true_ids.shape[0]
    acc_k = 0.0
    rec_m = 0.0
    for t in range(N):
        tr = set(int(v) for v in true_ids[t, :k])
        acc_k += len(tr & set(int(v) for v in pred_ids[t, :k])) / k
        rec_m += len(tr & set(int(v) for v in pred_ids[t])) / k
    return acc_k / N, rec_m / N


def prefill_set_accuracy(pred_ids, true_ids):
    """Prefill metric: |U pred ∩ U true| / |U true| over the layer's expert sets."""
    up = set(int(v) for v in np.asarray(pred_ids).ravel())
    ut = set(int(v) for v in np.asarray(true_ids).ravel())
    return len(up & ut) / max(1, len(ut))
