"""Shared glue of the GPU parity tests: move seeded inputs to both sides."""
import numpy as np
import torch

from oracle import moe as O
import paper_2502_12224_amd.binding as B
from workloads import gen_expert, gen_gate, gen_hidden, gen_shared_gate

DEV = "cuda"


def f32(t):
    return t.detach().to("cpu", torch.float32).numpy()


def oracle_expert(ex):
    ex = ex.cpu()
    z = {} if ex.z1 is None else dict(z1=ex.z1.numpy(), z3=ex.z3.numpy(), z2=ex.z2.numpy())
    return O.OracleExpert(ex.w1.numpy(), ex.s1.numpy(), ex.w3.numpy(), ex.s3.numpy(), ex.w2.numpy(),
                          ex.s2.numpy(), ex.bits, ex.group, **z)


def bias_np(b):
    return None if b is None else b.cpu().numpy()


def gpu_route(x, Wg, bias, k, renorm, want_probs=True):
    N, E = x.shape[0], Wg.shape[0]
    ids = torch.empty(N, k, dtype=torch.int32, device=DEV)
    w = torch.empty(N, k, dtype=torch.float32, device=DEV)
    probs = torch.empty(N, E, dtype=torch.float32, device=DEV) if want_probs else None
    B.fate_gate_route(x, Wg, bias, k, renorm, ids, w, probs)
    return ids, w, probs


def gpu_predict(x, Wg, bias, k, m):
    N, E = x.shape[0], Wg.shape[0]
    ids = torch.empty(N, m, dtype=torch.int32, device=DEV)
    w = torch.empty(N, m, dtype=torch.float32, device=DEV)
    pop = torch.full((E,), -7, dtype=torch.int32, device=DEV)
    B.fate_cross_layer_predict(x, Wg, bias, k, m, ids, w, pop)
    return ids, w, pop


def gpu_permute(ids, E):
    N, k = ids.shape
    P = N * k
    counts = torch.empty(E, dtype=torch.int32, device=DEV)
    offsets = torch.empty(E + 1, dtype=torch.int32, device=DEV)
    perm = torch.empty(max(P, 1), dtype=torch.int32, device=DEV)
    inv = torch.empty(max(P, 1), dtype=torch.int32, device=DEV)
    order = torch.empty(E, dtype=torch.int32, device=DEV)
    B.fate_permute(ids, E, counts, offsets, perm, inv, order)
    return counts, offsets, perm[:P], inv[:P], order


def check_routing(ids_gpu, w_gpu, ids_ref, w_ref, z_ref, kk, what=""):
    """ids exact outside near-tie rows; weights within 1e-6 + 1e-5*|ref|."""
    ids_gpu = ids_gpu.cpu().numpy()
    w_gpu = w_gpu.cpu().numpy().astype(np.float64)
    ties = set(O.near_tie_rows(z_ref, kk).tolist())
    rows = [t for t in range(ids_ref.shape[0]) if t not in ties]
    assert np.array_equal(ids_gpu[rows], ids_ref[rows]), what
    err = np.abs(w_gpu[rows] - w_ref[rows])
    assert (err <= 1e-6 + 1e-5 * np.abs(w_ref[rows])).all(), (what, err.max())
    for t in ties:   # a near-tie row may pick any expert within the margin of the k-th logit
        kth = np.sort(z_ref[t])[::-1][kk - 1]
        assert all(z_ref[t][e] >= kth - 1e-4 for e in ids_gpu[t]), what
        assert len(set(ids_gpu[t].tolist())) == kk
    return len(ties)


class GpuLayer:
    """Packed experts of one layer on the device plus their pointer tables."""

    def __init__(self, cfg, layer, experts=None, device=DEV):
        self.cfg = cfg
        want = range(cfg.E) if experts is None else experts
        self.host = {}
        self.packed = {}
        structs = []
        for e in range(cfg.E):
            if e in want:
                ex = gen_expert(cfg, layer, e, device=device)
                self.host[e] = ex
                self.packed[e] = B.PackedExpert(ex, device)
                structs.append(self.packed[e].struct())
            else:
                structs.append(B.fate_qexpert(0, 0, 0, 0, 0, 0, cfg.bits, cfg.group, cfg.I, 0))
        self.table = B.expert_table(structs, device)
        self.shared_host = [gen_expert(cfg, layer, s, shared=True, device=device) for s in range(cfg.n_shared)]
        self.shared_packed = [B.PackedExpert(ex, device) for ex in self.shared_host]
        self.shared_table = B.expert_table([p.struct() for p in self.shared_packed], device) if cfg.n_shared else None
        self.shared_gate = gen_shared_gate(cfg, layer, device)

    def desc(self, N, mode=0, y_is_fp32=True):
        c = self.cfg
        return B.make_ffn_desc(N, c.H, c.E, c.k, c.I, c.bits, c.group, c.n_shared, c.I_shared or 0, c.shared_bits,
                               c.group, y_is_fp32, mode)

    def ffn(self, x, counts, offsets, perm, inv_perm, order, topk_w, mode=0, y_is_fp32=True, ws_fill=0):
        N = x.shape[0]
        d = self.desc(N, mode, y_is_fp32)
        ws = torch.full((B.fate_moe_ffn_q_workspace(d),), ws_fill, dtype=torch.uint8, device=x.device)
        ws[:256] = 0                # the status word starts at zero
        y = torch.full((N, self.cfg.H), float("nan"), dtype=torch.float32 if y_is_fp32 else torch.bfloat16,
                       device=x.device)
        B.fate_moe_ffn_q(d, x, self.table, counts, offsets, perm, inv_perm, order, topk_w, self.shared_table,
                         self.shared_gate, y, ws)
        torch.cuda.synchronize()
        return y, ws


def ffn_rel_err(y_gpu, y_ref):
    """Per token row: max_i |y_gpu - y_ref| / max_i |y_ref|."""
    y_gpu = np.asarray(y_gpu, dtype=np.float64)
    num = np.abs(y_gpu - y_ref).max(axis=1)
    den = np.abs(y_ref).max(axis=1)
    return num / den
