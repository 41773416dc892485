"""The 2-bit expert copies of section 4.5 on the device: packing, both FFN paths on experts stored at
2 bits, and a layer that mixes 2- and 4-bit copies (what the popularity-aware hybrid transfer leaves in
the expert table), against the fp64 oracle working on the same stored copies.  Bar: 2e-3 per token row.
The quantisation error itself (against the unquantised weights) is printed, not graded."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import moe as O
import paper_2502_12224_amd.binding as B
from workloads import SHAPES, gen_expert, gen_expert_unquantized, gen_gate, gen_hidden, gen_shared_gate, quantize_sym
from helpers import DEV, bias_np, f32, ffn_rel_err, gpu_permute, oracle_expert

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _expected_int2_tiles(codes, rows, K):
    """The documented device-native layout written out with numpy: tile of 32 rows x 128 columns, lane =
    half * 32 + row, dword d of a lane = columns 16d .. 16d+15 of its 64, column 2i in bits 2i..2i+1 and
    column 2i+1 in bits 16+2i.."""
    u = ((O.unpack_codes(codes, 2) + 3) // 2).astype(np.uint32)
    out = np.zeros((rows // 32, K // 128, 64, 4), dtype=np.uint32)
    blk = u.reshape(rows // 32, 32, K // 128, 128)
    for half in range(2):
        for d in range(4):
            cols = blk[:, :, :, half * 64 + 16 * d: half * 64 + 16 * d + 16]        # rb, n, kb, 16
            word = np.zeros(cols.shape[:3], dtype=np.uint32)
            for i in range(8):
                word |= cols[..., 2 * i] << (2 * i)
                word |= cols[..., 2 * i + 1] << (2 * i + 16)
            out[:, :, half * 32:(half + 1) * 32, d] = word.transpose(0, 2, 1)
    return out.reshape(-1)


@pytest.mark.parametrize("rows,K", [(32, 128), (96, 512), (1408, 2048)])
def test_pack_weight_layout_int2(rows, K):
    g = torch.Generator().manual_seed(rows + K)
    w = torch.randn(rows, K, generator=g) * 0.02
    codes, _ = quantize_sym(w, 2, 128)
    src = codes.to(DEV)
    dst = torch.zeros_like(src)
    B.fate_pack_weight(src, rows, K, 2, dst)
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy().reshape(-1).view(np.uint32), _expected_int2_tiles(codes.numpy(), rows, K))


class MixedLayer:
    """Expert table of one layer whose routed experts are stored at the widths in `bits_of` (default 4)."""

    def __init__(self, cfg, layer, used, bits_of, zero_points=()):
        self.cfg = cfg
        self.host, self.packed, structs = {}, {}, []
        for e in range(cfg.E):
            if e in used:
                ex = gen_expert(cfg, layer, e, device=DEV, bits=bits_of.get(e, cfg.bits), group=128,
                                zero_points=e in zero_points)
                self.host[e] = ex
                self.packed[e] = B.PackedExpert(ex, DEV)
                structs.append(self.packed[e].struct())
            else:
                structs.append(B.fate_qexpert(0, 0, 0, 0, 0, 0, cfg.bits, cfg.group, cfg.I, 0))
        self.table = B.expert_table(structs, DEV)
        self.shared_host = [gen_expert(cfg, layer, s, shared=True, device=DEV) for s in range(cfg.n_shared)]
        self.shared_packed = [B.PackedExpert(ex, DEV) for ex in self.shared_host]
        self.shared_table = B.expert_table([p.struct() for p in self.shared_packed], DEV) if cfg.n_shared else None
        self.shared_gate = gen_shared_gate(cfg, layer, DEV)

    def ffn(self, x, ids, w, mode):
        c = self.cfg
        N = x.shape[0]
        d = B.make_ffn_desc(N, c.H, c.E, c.k, c.I, c.bits, c.group, c.n_shared, c.I_shared or 0, c.shared_bits, c.group,
                            True, mode)
        ws = torch.zeros(B.fate_moe_ffn_q_workspace(d), dtype=torch.uint8, device=DEV)
        y = torch.full((N, c.H), float("nan"), dtype=torch.float32, device=DEV)
        g = gpu_permute(ids, c.E)
        B.fate_moe_ffn_q(d, x, self.table, *g, w, self.shared_table, self.shared_gate, y, ws)
        torch.cuda.synchronize()
        return y, int(ws[:4].view(torch.int32)[0])

    def oracle(self, x, ids, w):
        experts = {e: oracle_expert(h) for e, h in self.host.items()}
        shared = [oracle_expert(h) for h in self.shared_host]
        sg = None if self.shared_gate is None else f32(self.shared_gate)
        return O.moe_ffn_grouped(f32(x), ids, w, experts, shared, sg)


def _route(cfg, N, layer=0):
    x = gen_hidden(cfg, N, device=DEV)
    Wg, b = gen_gate(cfg, layer, device=DEV)
    rid, rw, _, _ = O.gate_route(f32(x), f32(Wg), bias_np(b), cfg.k, cfg.renorm)
    return x, rid, rw


@pytest.mark.parametrize("name,N,mode,which", [
    ("tiny128", 40, 2, "all"), ("tiny128", 5, 1, "all"), ("tiny128", 200, 2, "odd"), ("tiny128", 7, 1, "odd"),
    ("qwen", 96, 2, "all"), ("qwen", 3, 1, "all"), ("qwen_prefill", 512, 2, "quarter"), ("qwen", 6, 1, "odd"),
    ("mixtral", 64, 2, "odd"),
])
def test_ffn_on_two_bit_and_mixed_width_experts(name, N, mode, which):
    """mode 2 = matrix-core path, 1 = decode kernels.  which: all routed experts at 2 bits, the odd ones, or the
    least popular quarter of the activated ones (the hybrid rule of section 4.5 applied to the true counts)."""
    cfg = dataclasses.replace(SHAPES["tiny"], name="tiny128", bits=4, group=128) if name == "tiny128" else SHAPES[name]
    x, rid, rw = _route(cfg, N)
    used = sorted(set(rid.ravel().tolist()))
    counts = np.bincount(rid.ravel(), minlength=cfg.E)
    if which == "all":
        low = set(used)
    elif which == "odd":
        low = {e for e in used if e % 2}
    else:
        by_pop = sorted(used, key=lambda e: (-counts[e], e))
        low = set(by_pop[len(by_pop) - len(by_pop) // 4:])
    L = MixedLayer(cfg, 0, used, {e: 2 for e in low})
    ids_d = torch.from_numpy(rid).to(DEV)
    w_d = torch.from_numpy(rw.astype(np.float32)).to(DEV)
    y, status = L.ffn(x, ids_d, w_d, mode)
    assert status == 0
    y_ref = L.oracle(x, rid, w_d.cpu().numpy().astype(np.float64))
    err = ffn_rel_err(f32(y), y_ref)
    print(f"{name} N={N} mode {mode}: {len(low)} of {len(used)} activated experts at 2 bits, max row error {err.max():.2e}",
          flush=True)
    assert np.isfinite(f32(y)).all() and err.max() <= TOL


def test_quantisation_error_of_the_hybrid_is_reported():
    """Not a parity check: the error the stored formats themselves cost against the unquantised weights, for
    all-4-bit experts, the hybrid with the least popular quarter at 2 bits, and all-2-bit experts (the reported
    counterpart of the paper's accuracy-vs-INT2-share figure, section 4.5)."""
    cfg = SHAPES["qwen_prefill"]
    N = 256
    x, rid, rw = _route(cfg, N)
    used = sorted(set(rid.ravel().tolist()))
    counts = np.bincount(rid.ravel(), minlength=cfg.E)
    by_pop = sorted(used, key=lambda e: (-counts[e], e))
    xn = f32(x).astype(np.float64)
    # fp64 reference on the unquantised weights (routed part only: the shared expert is the same in all three)
    y_fp = np.zeros((N, cfg.H))
    for e in used:
        W1, W3, W2 = (t.double().cpu().numpy() for t in gen_expert_unquantized(cfg, 0, e, device=DEV))
        t_idx, j_idx = np.nonzero(rid == e)
        h = O.silu(xn[t_idx] @ W1.T) * (xn[t_idx] @ W3.T)
        np.add.at(y_fp, t_idx, rw[t_idx, j_idx][:, None] * (h @ W2.T))
    out = {}
    for label, low in (("all 4-bit", set()), ("hybrid 25 %", set(by_pop[len(by_pop) - len(by_pop) // 4:])),
                       ("all 2-bit", set(used))):
        experts = {e: oracle_expert(gen_expert(cfg, 0, e, device=DEV, bits=2 if e in low else 4, group=128)) for e in used}
        y_q = O.moe_ffn_grouped(xn, rid, rw, experts)
        rel = np.linalg.norm(y_q - y_fp) / np.linalg.norm(y_fp)
        tokens_low = sum(int(counts[e]) for e in low) / counts.sum()
        out[label] = rel
        print(f"{label:12s}: {len(low):2d} of {len(used)} experts at 2 bits ({100 * tokens_low:.1f} % of the token-expert "
              f"pairs), relative error of the routed output vs unquantised weights {rel:.4f}", flush=True)
    assert out["all 4-bit"] < out["hybrid 25 %"] < out["all 2-bit"]
