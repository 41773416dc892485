"""Harness for a synthetic MoE layer stack: owns the device tensors and calls
the libfate entry points in order.  No arithmetic of the method lives here;
the residual / normalisation glue that chains layers (h += y, x = bf16(h /
rms(h))) comes from the workload module and is harness-only.
"""
import ctypes as C

import torch

from . import binding as B
from workloads import (MoEShape, chain_next_hidden, gen_expert, gen_gate, gen_hidden, gen_shared_gate,
                       unit_rmsnorm_bf16)


class LayerWeights:
    def __init__(self, cfg: MoEShape, layer: int, device, experts=None):
        self.Wg, self.bias = gen_gate(cfg, layer, device)
        self.shared_gate = gen_shared_gate(cfg, layer, device)
        self.packed = {}
        structs = []
        want = range(cfg.E) if experts is None else experts
        for e in range(cfg.E):
            if e in want:
                pe = B.PackedExpert(gen_expert(cfg, layer, e, device=device), device)
                self.packed[e] = pe
                structs.append(pe.struct())
            else:
                structs.append(B.fate_qexpert(0, 0, 0, 0, 0, 0, cfg.bits, cfg.group, cfg.I, 0))
        self.table = B.expert_table(structs, device)
        self.shared = [B.PackedExpert(gen_expert(cfg, layer, s, shared=True, device=device), device)
                       for s in range(cfg.n_shared)]
        self.shared_table = B.expert_table([p.struct() for p in self.shared], device) if cfg.n_shared else None

    def nbytes(self):
        return sum(p.nbytes() for p in self.packed.values()) + sum(p.nbytes() for p in self.shared)


class LayerBuffers:
    """Outputs of the routing calls and the FFN for one layer and N tokens."""

    def __init__(self, cfg: MoEShape, N: int, device, mode=0):
        E, k, m, H = cfg.E, cfg.k, cfg.m, cfg.H
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.ids = torch.zeros(N, k, **i32)
        self.w = torch.zeros(N, k, **f32)
        self.pred_ids = torch.zeros(N, m, **i32)
        self.pred_w = torch.zeros(N, m, **f32)
        self.pred_pop = torch.zeros(E, **i32)
        self.counts = torch.zeros(E, **i32)
        self.offsets = torch.zeros(E + 1, **i32)
        self.perm = torch.zeros(max(N * k, 1), **i32)
        self.inv_perm = torch.zeros(max(N * k, 1), **i32)
        self.order = torch.zeros(E, **i32)
        self.y = torch.zeros(N, H, **f32)
        self.desc = B.make_ffn_desc(N, H, E, k, cfg.I, cfg.bits, cfg.group, cfg.n_shared, cfg.I_shared or 0,
                                    cfg.shared_bits, cfg.group, True, mode)
        self.ffn_ws = torch.zeros(B.fate_moe_ffn_q_workspace(self.desc), dtype=torch.uint8, device=device)
        self.fused_ok = 1 <= N <= 16
        self.route_ws = torch.zeros(B.fate_route_fused_workspace(max(N, 1), E), dtype=torch.uint8, device=device)


def layer_forward(cfg: MoEShape, lw: LayerWeights, lw_next, x, buf: LayerBuffers, fused=None, phases=0):
    """One MoE layer: route, predict the next layer's experts, permute, FFN."""
    fused = buf.fused_ok if fused is None else fused
    if fused:
        B.fate_route_fused(x, lw.Wg, lw.bias, None if lw_next is None else lw_next.Wg,
                           None if lw_next is None else lw_next.bias, cfg.k, cfg.m, cfg.renorm, buf.ids, buf.w,
                           buf.pred_ids, buf.pred_w, buf.pred_pop, buf.counts, buf.offsets, buf.perm,
                           buf.inv_perm, buf.order, buf.route_ws)
    else:
        B.fate_gate_route(x, lw.Wg, lw.bias, cfg.k, cfg.renorm, buf.ids, buf.w, None)
        if lw_next is not None:
            B.fate_cross_layer_predict(x, lw_next.Wg, lw_next.bias, cfg.k, cfg.m, buf.pred_ids, buf.pred_w,
                                       buf.pred_pop)
        B.fate_permute(buf.ids, cfg.E, buf.counts, buf.offsets, buf.perm, buf.inv_perm, buf.order)
    buf.desc.phases = phases
    B.fate_moe_ffn_q(buf.desc, x, lw.table, buf.counts, buf.offsets, buf.perm, buf.inv_perm, buf.order, buf.w,
                     lw.shared_table, lw.shared_gate, buf.y, buf.ffn_ws)
    return buf.y


class MoEStack:
    """All layers of a synthetic stack resident on the device."""

    def __init__(self, cfg: MoEShape, device="cuda", layers=None, progress=None):
        self.cfg = cfg
        self.device = device
        self.nl = cfg.layers if layers is None else layers
        self.layers = []
        for l in range(self.nl):
            self.layers.append(LayerWeights(cfg, l, device))
            if progress:
                progress(l)

    def nbytes(self):
        return sum(l.nbytes() for l in self.layers)

    def chain(self, N, steps, bufs=None):
        """Free-running chained pass (untimed use): returns the gate inputs
        x[step][layer] and the true / predicted ids for accuracy statistics."""
        cfg = self.cfg
        bufs = bufs or LayerBuffers(cfg, N, self.device)
        xs, true_ids, pred_ids = [], [], []
        for s in range(steps):
            h = gen_hidden(cfg, N, step=s, device=self.device).to(torch.float32)
            xs_s, t_s, p_s = [], [], []
            for l in range(self.nl):
                x = unit_rmsnorm_bf16(h)
                nxt = self.layers[l + 1] if l + 1 < self.nl else None
                y = layer_forward(cfg, self.layers[l], nxt, x, bufs)
                xs_s.append(x)
                t_s.append(bufs.ids.clone())
                p_s.append(bufs.pred_ids.clone())
                h = chain_next_hidden(h, y)
            xs.append(torch.stack(xs_s))
            true_ids.append(torch.stack(t_s))
            pred_ids.append(torch.stack(p_s))
        return torch.stack(xs), torch.stack(true_ids), torch.stack(pred_ids)
