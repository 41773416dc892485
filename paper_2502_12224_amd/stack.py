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
        self.fused_ok = 1 <= N <= 16 or (N >= 64 and cfg.H % 1024 == 0)
        self.route_ws = torch.zeros(B.fate_route_fused_workspace(max(N, 1), E), dtype=torch.uint8, device=device)
        # whole layer in one launch (small decode batches)
        self.one_launch_ok = 1 <= N <= 8 and N * k <= 64 and mode != 2
        if self.one_launch_ok:
            nbytes, self.status_offset = B.fate_moe_layer_decode_workspace(self.desc)
            self.layer_ws = torch.zeros(nbytes, dtype=torch.uint8, device=device)

    def status(self):
        """Status word of the last one-launch layer call (0 = fine)."""
        return int(self.layer_ws[self.status_offset:self.status_offset + 4].view(torch.int32)[0])


def layer_forward(cfg: MoEShape, lw: LayerWeights, lw_next, x, buf: LayerBuffers, fused=None, one_launch=None,
                  hint_ids=None):
    """One MoE layer: route, predict the next layer's experts, permute, FFN.
    hint_ids: the previous layer's prediction for this layer (device int32, k ids), or None."""
    one_launch = (buf.one_launch_ok and fused is None) if one_launch is None else one_launch
    if one_launch:
        B.fate_moe_layer_decode(buf.desc, x, lw.Wg, lw.bias, None if lw_next is None else lw_next.Wg,
                                None if lw_next is None else lw_next.bias, cfg.m, cfg.renorm, buf.ids, buf.w,
                                buf.pred_ids, buf.pred_w, buf.pred_pop, buf.counts, buf.offsets, buf.perm,
                                buf.inv_perm, buf.order, lw.table, lw.shared_table, lw.shared_gate, buf.y,
                                buf.layer_ws, hint_ids=hint_ids)
        return buf.y
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


def _align(v, a=256):
    return (v + a - 1) // a * a


class OffloadedStack:
    """Stack whose routed experts live in a pinned host pool; a device slot
    pool holds the cached / staged ones.  Drives fate_expert_cache_step with
    the built-in HIP copy engine (side stream) around the per-layer calls."""

    def __init__(self, cfg: MoEShape, cache_total, n_max, staging_slots, device="cuda", layers=None,
                 L_shallow=None, progress=None, predictor="gate", low_bits=0):
        """predictor: "gate" = the cross-layer gate prediction (the method), "eap" = the activation-path
        baseline (co-activation statistics, fed through eap_observe), "none" = no prediction.
        low_bits: 2 = also keep a 2-bit copy of every routed expert in a second pinned pool (section 4.5:
        both widths live in host memory); set_low_percent() then switches the hybrid transfer width on."""
        self.cfg, self.device = cfg, device
        self.predictor = predictor
        # >0: a prefill layer's FFN runs in pieces that follow the cache step's compute order - experts
        # found in the cache first (with the shared experts), then the prefetched and the demand-loaded
        # ones `overlap_piece` at a time, each piece waiting only for its own transfers
        self.overlap_piece = 0
        self.nl = cfg.layers if layers is None else layers
        L, E = self.nl, cfg.E
        lib = B.lib()
        self.lib = lib
        # slot layout: the six arrays of one expert, 256-byte aligned
        wb = cfg.I * cfg.H * cfg.bits // 8
        sb = cfg.I * cfg.H // cfg.group * 2
        off, offs = 0, {}
        for name, nb in (("w1", wb), ("w3", wb), ("w2", wb), ("s1", sb), ("s3", sb), ("s2", sb)):
            offs[name] = off
            off = _align(off + nb)
        self.slot_bytes = off
        self.layout = B.fate_slot_layout(self.slot_bytes, offs["w1"], offs["w3"], offs["w2"], offs["s1"], offs["s3"],
                                         offs["s2"], cfg.bits, cfg.group, cfg.I)
        # dense parts stay on the device: gates, shared experts
        self.gates, self.shared, self.shared_tables, self.shared_gates = [], [], [], []
        self.host_pool = torch.empty(L * E, self.slot_bytes, dtype=torch.uint8, pin_memory=True)
        stage = torch.zeros(self.slot_bytes, dtype=torch.uint8, device=device)
        self.low_bits = low_bits
        if low_bits:
            assert low_bits == 2 and cfg.group % 128 == 0 and cfg.H % 128 == 0 and cfg.I % 128 == 0
            wl = cfg.I * cfg.H * low_bits // 8
            offl, o = {}, 0
            for name, nb in (("w1", wl), ("w3", wl), ("w2", wl), ("s1", sb), ("s3", sb), ("s2", sb)):
                offl[name] = o
                o = _align(o + nb)
            self.low_slot_bytes = o
            self.low_layout = B.fate_slot_layout(o, offl["w1"], offl["w3"], offl["w2"], offl["s1"], offl["s3"],
                                                 offl["s2"], low_bits, cfg.group, cfg.I)
            self.host_pool_low = torch.empty(L * E, o, dtype=torch.uint8, pin_memory=True)
            stage_low = torch.zeros(o, dtype=torch.uint8, device=device)
        for l in range(L):
            self.gates.append(gen_gate(cfg, l, device))
            self.shared_gates.append(gen_shared_gate(cfg, l, device))
            sh = [B.PackedExpert(gen_expert(cfg, l, s, shared=True, device=device), device) for s in range(cfg.n_shared)]
            self.shared.append(sh)
            self.shared_tables.append(B.expert_table([p.struct() for p in sh], device) if cfg.n_shared else None)
            for e in range(E):
                pe = B.PackedExpert(gen_expert(cfg, l, e, device=device), device)
                for name in offs:
                    t = pe.t[name].reshape(-1).view(torch.uint8)
                    stage[offs[name]:offs[name] + t.numel()] = t
                self.host_pool[l * E + e].copy_(stage)
                if low_bits:
                    pl = B.PackedExpert(gen_expert(cfg, l, e, device=device, bits=low_bits), device)
                    for name in offl:
                        t = pl.t[name].reshape(-1).view(torch.uint8)
                        stage_low[offl[name]:offl[name] + t.numel()] = t
                    self.host_pool_low[l * E + e].copy_(stage_low)
            if progress:
                progress(l)
        torch.cuda.synchronize()
        self.copy_stream = torch.cuda.Stream()
        self.compute_stream = torch.cuda.current_stream()
        caps = (C.c_int32 * L)()
        Ls = cfg.L_shallow if L_shallow is None else L_shallow
        lib.fate_cache_layer_capacities(L, E, cache_total, Ls, caps)
        self.caps = list(caps)
        self.total_slots = sum(self.caps) + staging_slots
        self.slot_pool = torch.zeros(self.total_slots, self.slot_bytes, dtype=torch.uint8, device=device)
        self.table = torch.zeros(L * E * C.sizeof(B.fate_qexpert), dtype=torch.uint8, device=device)
        self.engine = lib.fate_hip_engine_create(L, E, self.total_slots, C.byref(self.layout),
                                                 C.c_void_p(self.slot_pool.data_ptr()),
                                                 C.c_void_p(self.host_pool.data_ptr()),
                                                 C.c_void_p(self.table.data_ptr()),
                                                 C.c_void_p(self.copy_stream.cuda_stream),
                                                 C.c_void_p(self.compute_stream.cuda_stream))
        if not self.engine:
            raise B.FateError(6, lib.fate_last_error().decode())
        self._copy_fn = B.COPY_FN(("fate_hip_engine_copy", lib))
        self.cache = lib.fate_cache_create(L, E, cache_total, Ls, n_max, staging_slots, self._copy_fn,
                                           C.c_void_p(self.engine))
        assert lib.fate_cache_total_slots(self.cache) == self.total_slots
        B._check(lib.fate_cache_set_low_precision(self.cache, 0, cfg.bits, 2))     # width labels of the load list
        if low_bits:
            B._check(lib.fate_hip_engine_set_low_pool(self.engine, C.byref(self.low_layout),
                                                      C.c_void_p(self.host_pool_low.data_ptr())))
        for l in range(L):
            for e in range(E):
                s = lib.fate_cache_slot_of(self.cache, l, e)
                if s >= 0:
                    B._check(lib.fate_hip_engine_preload(self.engine, l, e, s))
        self.done_event = torch.cuda.Event()
        self.have_done = False
        self.stats = dict(hit_cache=0, hit_prefetch=0, miss=0, pair_hits=0, pair_misses=0, prefetch=0, wasted=0,
                          evicted=0)
        self.trace = []          # per step: (layer, compute_order, loads) for checks against the oracle
        self.trace_bits = []     # per step: the width of every load
        self.piece_log = []      # overlapped prefill: (layer, [experts of each piece])
        self.keep_trace = False
        self._h_counts = torch.zeros(2, E, dtype=torch.int32).pin_memory()
        self._h_ids = torch.zeros(4096 * cfg.k, dtype=torch.int32).pin_memory()
        self.eap = lib.fate_eap_create(L, E) if predictor == "eap" else None
        self._eap_prev = None          # (layer, host ids) of the previous layer call, for the statistics
        self.eap_learning = False
        self._order = (C.c_int32 * E)()
        self._slots = (C.c_int32 * E)()
        self._loads = (B.fate_cache_load * 512)()
        self._st = B.fate_cache_stats()
        self._nact = C.c_int32(0)

    def set_low_percent(self, percent):
        """Popularity-aware hybrid transfer width (section 4.5): the least popular `percent` % of the experts
        predicted for the next layer travel as low-width copies.  A caller sets it for prefill, 0 for decode."""
        assert percent == 0 or self.low_bits
        B._check(self.lib.fate_cache_set_low_precision(self.cache, percent, self.cfg.bits, self.low_bits or 2))

    def table_for(self, l):
        return self.table[l * self.cfg.E * C.sizeof(B.fate_qexpert):]

    def layer(self, l, x, buf: LayerBuffers):
        """Route, predict, permute, cache step (with copies), FFN for layer l."""
        cfg, lib = self.cfg, self.lib
        nxt = l + 1 < self.nl
        Wg, bias = self.gates[l]
        Wg2, bias2 = self.gates[l + 1] if nxt else (None, None)
        if buf.fused_ok:
            B.fate_route_fused(x, Wg, bias, Wg2, bias2, cfg.k, cfg.m, cfg.renorm, buf.ids, buf.w, buf.pred_ids,
                               buf.pred_w, buf.pred_pop, buf.counts, buf.offsets, buf.perm, buf.inv_perm, buf.order,
                               buf.route_ws)
        else:
            B.fate_gate_route(x, Wg, bias, cfg.k, cfg.renorm, buf.ids, buf.w, None)
            if nxt:
                B.fate_cross_layer_predict(x, Wg2, bias2, cfg.k, cfg.m, buf.pred_ids, buf.pred_w, buf.pred_pop)
            B.fate_permute(buf.ids, cfg.E, buf.counts, buf.offsets, buf.perm, buf.inv_perm, buf.order)
        # the host needs the routing result to check residency (the one device -> host hop per layer)
        self._h_counts[0].copy_(buf.counts, non_blocking=True)
        if nxt and self.predictor == "gate":
            self._h_counts[1].copy_(buf.pred_pop, non_blocking=True)
        nk = buf.ids.numel()
        if self.eap is not None:
            self._h_ids[:nk].copy_(buf.ids.reshape(-1), non_blocking=True)
        torch.cuda.current_stream().synchronize()
        if self.eap is not None:
            N = nk // cfg.k
            if self.eap_learning and self._eap_prev is not None and self._eap_prev[0] == l - 1 and \
                    self._eap_prev[1].numel() == nk:
                B._check(lib.fate_eap_update(self.eap, l - 1, C.c_void_p(self._eap_prev[1].data_ptr()),
                                             C.c_void_p(self._h_ids.data_ptr()), N, cfg.k))
            self._eap_prev = (l, self._h_ids[:nk].clone())
            if nxt:
                B._check(lib.fate_eap_predict(self.eap, l, C.c_void_p(self._h_ids.data_ptr()), N, cfg.k, cfg.m,
                                              C.c_void_p(self._h_counts[1].data_ptr())))
        have_pred = nxt and self.predictor in ("gate", "eap")
        B._check(lib.fate_hip_engine_begin_step(self.engine, C.c_void_p(self.done_event.cuda_event)
                                                if self.have_done else None))
        st = self._st
        B._check(lib.fate_expert_cache_step_dense(self.cache, l, C.c_void_p(self._h_counts[0].data_ptr()),
                                                  C.c_void_p(self._h_counts[1].data_ptr()) if have_pred else None,
                                                  self._order, self._slots, C.byref(self._nact), self._loads, 512,
                                                  C.byref(st)))
        n = self._nact.value
        pieces = None
        if self.overlap_piece > 0 and buf.desc.mode == 2 or (self.overlap_piece > 0 and buf.desc.mode == 0 and x.shape[0] > 16):
            nc = st.n_hit_cache
            pieces = [(0, nc)] + [(i, min(n, i + self.overlap_piece)) for i in range(nc, n, self.overlap_piece)]
        else:
            B._check(lib.fate_hip_engine_wait_ready(self.engine, self._slots, n))
        s = self.stats
        s["hit_cache"] += st.n_hit_cache; s["hit_prefetch"] += st.n_hit_prefetch; s["miss"] += st.n_miss
        s["pair_hits"] += st.pair_hits; s["pair_misses"] += st.pair_misses; s["prefetch"] += st.n_prefetch_issued
        s["wasted"] += st.n_wasted; s["evicted"] += st.n_evicted
        if self.keep_trace:
            self.trace.append((l, list(self._order[:n]), [(ld.layer, ld.expert, ld.slot, bool(ld.demand))
                                                          for ld in self._loads[:min(st.n_loads, 512)]]))
            self.trace_bits.append([ld.bits for ld in self._loads[:min(st.n_loads, 512)]])
        if pieces is None:
            B.fate_moe_ffn_q(buf.desc, x, self.table_for(l), buf.counts, buf.offsets, buf.perm, buf.inv_perm, buf.order,
                             buf.w, self.shared_tables[l], self.shared_gates[l], buf.y, buf.ffn_ws)
        else:
            self.piece_log.append((l, [list(self._order[a:b]) for a, b in pieces]))
            for i, (a, b) in enumerate(pieces):
                if b > a:
                    sl = (C.c_int32 * (b - a))(*self._slots[a:b])
                    B._check(lib.fate_hip_engine_wait_ready(self.engine, sl, b - a))
                B.fate_moe_ffn_q_part(buf.desc, x, self.table_for(l), buf.counts, buf.offsets, buf.perm, buf.inv_perm,
                                      buf.order, buf.w, self.shared_tables[l], self.shared_gates[l], buf.y, buf.ffn_ws,
                                      list(self._order[a:b]), first=i == 0, last=i == len(pieces) - 1)
        self.done_event.record()
        self.have_done = True
        return buf.y

    def bytes_copied(self):
        return self.lib.fate_hip_engine_bytes_copied(self.engine)

    def close(self):
        torch.cuda.synchronize()
        self.lib.fate_cache_destroy(self.cache)
        self.lib.fate_hip_engine_destroy(self.engine)
        if self.eap is not None:
            self.lib.fate_eap_destroy(self.eap)
