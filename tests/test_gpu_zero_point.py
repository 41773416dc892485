"""Experts stored with zero-points, w = (u - z) * s per group (the asymmetric format that HQQ-style
quantisers write, section 4.5): both FFN paths on such copies, alone and mixed with symmetric ones in one
layer, against the fp64 oracle working on the same stored fields, scales and zero-points.  Bar: 2e-3 per
token row.  One case takes its stored values from the oracle's own HQQ-style quantiser."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import moe as O
import paper_2502_12224_amd.binding as B
from workloads import SHAPES, QExpertHost, gen_expert_unquantized
from helpers import DEV, f32, ffn_rel_err, gpu_permute
from test_gpu_int2 import MixedLayer, _route

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _cfg(name):
    return dataclasses.replace(SHAPES["tiny"], name="tiny128", bits=4, group=128) if name == "tiny128" else SHAPES[name]


@pytest.mark.parametrize("name,N,mode,bits,which", [
    ("tiny128", 40, 2, 4, "all"), ("tiny128", 5, 1, 4, "all"), ("tiny128", 200, 2, 2, "all"), ("tiny128", 7, 1, 2, "all"),
    ("tiny128", 19, 1, 4, "odd"), ("tiny128", 64, 2, 2, "odd"),
    ("qwen", 96, 2, 4, "all"), ("qwen", 3, 1, 4, "all"), ("qwen", 8, 1, 2, "odd"), ("qwen_prefill", 512, 2, 2, "odd"),
    ("mixtral", 1, 1, 4, "all"), ("mixtral", 64, 2, 4, "odd"), ("deepseek", 8, 1, 4, "odd"),
])
def test_ffn_on_experts_with_zero_points(name, N, mode, bits, which):
    """mode 2 = matrix-core path, 1 = decode kernels; which: every activated routed expert carries zero-points, or
    the odd ones (the even ones stay symmetric 4-bit: both kinds in one launch)."""
    cfg = _cfg(name)
    x, rid, rw = _route(cfg, N)
    used = sorted(set(rid.ravel().tolist()))
    zp = set(used) if which == "all" else {e for e in used if e % 2}
    L = MixedLayer(cfg, 0, used, {e: bits for e in zp}, zero_points=zp)
    ids_d = torch.from_numpy(rid).to(DEV)
    w_d = torch.from_numpy(rw.astype(np.float32)).to(DEV)
    y, status = L.ffn(x, ids_d, w_d, mode)
    assert status == 0
    y_ref = L.oracle(x, rid, w_d.cpu().numpy().astype(np.float64))
    err = ffn_rel_err(f32(y), y_ref)
    print(f"{name} N={N} mode {mode}: {len(zp)} of {len(used)} activated experts with {bits}-bit fields and zero-points, "
          f"max row error {err.max():.2e}", flush=True)
    assert np.isfinite(f32(y)).all() and err.max() <= TOL


def _pack_fields(u, bits):
    u = torch.from_numpy(u.astype(np.uint8))
    if bits == 4:
        return (u[:, 0::2] | (u[:, 1::2] << 4)).contiguous()
    return (u[:, 0::4] | (u[:, 1::4] << 2) | (u[:, 2::4] << 4) | (u[:, 3::4] << 6)).contiguous()


@pytest.mark.parametrize("bits,mode,N", [(4, 1, 6), (4, 2, 48), (2, 1, 6), (2, 2, 48)])
def test_ffn_on_values_written_by_the_hqq_style_quantiser(bits, mode, N):
    """The stored fields, scales and refined zero-points come out of the oracle's quantiser (fractional
    zero-points, unlike the plain min / max ones), the device reads exactly those."""
    cfg = _cfg("tiny128")
    x, rid, rw = _route(cfg, N)
    used = sorted(set(rid.ravel().tolist()))
    host = {}
    for e in used:
        q = []
        for W in gen_expert_unquantized(cfg, 0, e):
            u, s, z = O.quantize_asym(W.double().numpy(), bits, 128, hqq_iters=8)
            q.append((_pack_fields(u, bits), torch.from_numpy(s), torch.from_numpy(z)))
        (w1, s1, z1), (w3, s3, z3), (w2, s2, z2) = q
        host[e] = QExpertHost(w1, w3, w2, s1, s3, s2, bits, 128, cfg.I, cfg.H, z1, z3, z2)
    L = MixedLayer(cfg, 0, [], {})
    L.host = host
    L.packed = {e: B.PackedExpert(h, DEV) for e, h in host.items()}
    structs = [L.packed[e].struct() if e in host else B.fate_qexpert(0, 0, 0, 0, 0, 0, cfg.bits, cfg.group, cfg.I, 0)
               for e in range(cfg.E)]
    L.table = B.expert_table(structs, DEV)
    ids_d = torch.from_numpy(rid).to(DEV)
    w_d = torch.from_numpy(rw.astype(np.float32)).to(DEV)
    y, status = L.ffn(x, ids_d, w_d, mode)
    assert status == 0
    err = ffn_rel_err(f32(y), L.oracle(x, rid, w_d.cpu().numpy().astype(np.float64)))
    print(f"HQQ-style {bits}-bit, mode {mode}: max row error {err.max():.2e}", flush=True)
    assert err.max() <= TOL


def test_eight_bit_entry_with_zero_points_is_flagged():
    """Zero-points exist for the 4- and 2-bit formats; an 8-bit entry that carries them is reported in the
    status word (bit 2) and contributes nothing, on both paths."""
    cfg = _cfg("tiny128")
    for mode, N in ((1, 4), (2, 40)):
        x, rid, rw = _route(cfg, N)
        used = sorted(set(rid.ravel().tolist()))
        L = MixedLayer(cfg, 0, used, {}, zero_points={used[0]})
        st = L.packed[used[0]].struct()
        st.bits = 8
        structs = [st if e == used[0] else (L.packed[e].struct() if e in L.packed else
                                            B.fate_qexpert(0, 0, 0, 0, 0, 0, cfg.bits, cfg.group, cfg.I, 0)) for e in range(cfg.E)]
        L.table = B.expert_table(structs, DEV)
        y, status = L.ffn(x, torch.from_numpy(rid).to(DEV), torch.from_numpy(rw.astype(np.float32)).to(DEV), mode)
        assert status & 4
        assert np.isfinite(f32(y)).all()
