"""ctypes binding of libfate: argument marshalling only.

Every function here has the name of the C entry point it calls (include/fate.h)
and does nothing but turn torch tensors into raw pointers and sizes.  All
arithmetic of the hot path runs in the HIP kernels of libfate.so; there is no
fallback: if the library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfate.so")

FATE_OK = 0
STATUS_NAMES = {0: "FATE_OK", 1: "FATE_EINVAL", 2: "FATE_ESHAPE", 3: "FATE_EALIGN", 4: "FATE_EWORKSPACE",
                5: "FATE_ENOTRESIDENT", 6: "FATE_EHIP", 7: "FATE_ECAPACITY"}

EXPORTS = [
    "fate_last_error", "fate_version", "fate_gate_route", "fate_cross_layer_predict", "fate_permute",
    "fate_route_fused_workspace", "fate_route_fused", "fate_pack_weight", "fate_pack_scales", "fate_moe_ffn_q_workspace",
    "fate_moe_ffn_q", "fate_moe_ffn_q_part", "fate_profile_ffn_mfma_phase", "fate_moe_layer_decode_workspace", "fate_moe_layer_decode",
    "fate_moe_layer_decode_noalloc", "fate_cache_total_from_budget", "fate_n_max_from_times", "fate_cache_layer_capacities",
    "fate_cache_create", "fate_cache_destroy", "fate_cache_total_slots", "fate_cache_set_n_max",
    "fate_cache_set_low_precision", "fate_hip_engine_set_low_pool", "fate_cache_slot_of",
    "fate_cache_resident", "fate_expert_cache_step", "fate_expert_cache_step_dense",
    "fate_expert_cache_step_layers", "fate_hip_engine_create", "fate_hip_engine_destroy",
    "fate_hip_engine_copy", "fate_hip_engine_begin_step", "fate_hip_engine_wait_ready",
    "fate_hip_engine_preload", "fate_hip_engine_bytes_copied",
    "fate_eap_create", "fate_eap_destroy", "fate_eap_update", "fate_eap_predict",
]


class FateError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {msg}")
        self.status = status


class fate_ffn_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "H", "E", "k", "I_max", "bits", "group", "n_shared",
                                         "I_shared_max", "shared_bits", "shared_group", "y_is_fp32", "mode",
                                         "reserved")]


class fate_qexpert(C.Structure):
    _fields_ = [("w1", C.c_void_p), ("w3", C.c_void_p), ("w2", C.c_void_p), ("s1", C.c_void_p),
                ("s3", C.c_void_p), ("s2", C.c_void_p), ("bits", C.c_int32), ("group", C.c_int32),
                ("I", C.c_int32), ("reserved", C.c_int32), ("z1", C.c_void_p), ("z3", C.c_void_p),
                ("z2", C.c_void_p), ("reserved2", C.c_int64)]


class fate_cache_stats(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_hit_cache", "n_hit_prefetch", "n_miss", "pair_hits", "pair_misses",
                                         "n_prefetch_issued", "n_prefetch_dropped", "n_wasted", "n_evicted",
                                         "n_loads")]


class fate_cache_load(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("layer", "expert", "slot", "demand", "bits")]


class fate_slot_layout(C.Structure):
    _fields_ = [("slot_bytes", C.c_size_t), ("off_w1", C.c_size_t), ("off_w3", C.c_size_t),
                ("off_w2", C.c_size_t), ("off_s1", C.c_size_t), ("off_s3", C.c_size_t), ("off_s2", C.c_size_t),
                ("bits", C.c_int32), ("group", C.c_int32), ("I", C.c_int32)]


COPY_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int)

_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2502_12224_amd.build). "
                "There is no fallback path.")
        L = C.CDLL(LIB_PATH)
        L.fate_last_error.restype = C.c_char_p
        L.fate_version.restype = C.c_char_p
        L.fate_cache_create.restype = C.c_void_p
        L.fate_cache_create.argtypes = [C.c_int] * 6 + [COPY_FN, C.c_void_p]
        L.fate_cache_destroy.argtypes = [C.c_void_p]
        L.fate_cache_destroy.restype = None
        L.fate_cache_total_slots.argtypes = [C.c_void_p]
        L.fate_cache_set_n_max.argtypes = [C.c_void_p, C.c_int]
        L.fate_cache_set_low_precision.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int]
        L.fate_hip_engine_set_low_pool.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.fate_cache_slot_of.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.fate_cache_resident.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.fate_cache_total_from_budget.restype = C.c_int64
        L.fate_cache_total_from_budget.argtypes = [C.c_int64] * 3
        L.fate_n_max_from_times.restype = C.c_int32
        L.fate_n_max_from_times.argtypes = [C.c_double] * 4
        L.fate_expert_cache_step.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                             C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                             C.c_void_p]
        L.fate_expert_cache_step_dense.argtypes = [C.c_void_p, C.c_int] + [C.c_void_p] * 6 + [C.c_int, C.c_void_p]
        L.fate_expert_cache_step_layers.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                                    C.c_void_p]
        L.fate_hip_engine_create.restype = C.c_void_p
        L.fate_hip_engine_create.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p]
        L.fate_hip_engine_destroy.argtypes = [C.c_void_p]
        L.fate_hip_engine_destroy.restype = None
        L.fate_hip_engine_begin_step.argtypes = [C.c_void_p, C.c_void_p]
        L.fate_hip_engine_wait_ready.argtypes = [C.c_void_p, C.c_void_p, C.c_int]
        L.fate_hip_engine_preload.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int]
        L.fate_hip_engine_bytes_copied.restype = C.c_uint64
        L.fate_hip_engine_bytes_copied.argtypes = [C.c_void_p]
        L.fate_eap_create.restype = C.c_void_p
        L.fate_eap_create.argtypes = [C.c_int, C.c_int]
        L.fate_eap_destroy.restype = None
        L.fate_eap_destroy.argtypes = [C.c_void_p]
        L.fate_eap_update.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int]
        L.fate_eap_predict.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        _lib = L
    return _lib


def _check(status):
    if status != FATE_OK:
        raise FateError(status, lib().fate_last_error().decode())


def _p(t):
    if t is None:
        return C.c_void_p(0)
    return C.c_void_p(t.data_ptr())


def _stream(stream=None):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def fate_version():
    return lib().fate_version().decode()


def fate_gate_route(x, Wg, bias, k, renorm, topk_ids, topk_w, probs=None, stream=None):
    N, H = x.shape
    E = Wg.shape[0]
    _check(lib().fate_gate_route(_stream(stream), _p(x), _p(Wg), _p(bias), N, H, E, k, int(renorm),
                                 _p(topk_ids), _p(topk_w), _p(probs)))


def fate_cross_layer_predict(x, Wg_next, bias_next, k, m, pred_ids, pred_w, pred_pop, stream=None):
    N, H = x.shape
    E = Wg_next.shape[0]
    _check(lib().fate_cross_layer_predict(_stream(stream), _p(x), _p(Wg_next), _p(bias_next), N, H, E, k, m,
                                          _p(pred_ids), _p(pred_w), _p(pred_pop)))


def fate_permute(topk_ids, E, counts, offsets, perm, inv_perm, expert_order, stream=None):
    N, k = topk_ids.shape
    _check(lib().fate_permute(_stream(stream), _p(topk_ids), N, k, E, _p(counts), _p(offsets), _p(perm),
                              _p(inv_perm), _p(expert_order)))


def fate_route_fused_workspace(N, E):
    b = C.c_size_t(0)
    _check(lib().fate_route_fused_workspace(N, E, C.byref(b)))
    return b.value


def fate_route_fused(x, Wg, bias, Wg_next, bias_next, k, m, renorm, topk_ids, topk_w, pred_ids, pred_w,
                     pred_pop, counts, offsets, perm, inv_perm, expert_order, workspace, stream=None):
    N, H = x.shape
    E = Wg.shape[0]
    _check(lib().fate_route_fused(_stream(stream), _p(x), _p(Wg), _p(bias), _p(Wg_next), _p(bias_next), N, H, E,
                                  k, m, int(renorm), _p(topk_ids), _p(topk_w), _p(pred_ids), _p(pred_w),
                                  _p(pred_pop), _p(counts), _p(offsets), _p(perm), _p(inv_perm),
                                  _p(expert_order), _p(workspace),
                                  C.c_size_t(workspace.numel() * workspace.element_size())))


def fate_pack_weight(canonical, rows, K, bits, packed, stream=None):
    _check(lib().fate_pack_weight(_stream(stream), _p(canonical), rows, K, bits, _p(packed)))


class fate_route_out(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("topk_ids", "topk_w", "pred_ids", "pred_w", "pred_pop", "counts",
                                          "offsets", "perm", "inv_perm", "expert_order")]


def fate_moe_layer_decode_workspace(desc):
    """(bytes, byte offset of the status word)."""
    b, o = C.c_size_t(0), C.c_size_t(0)
    _check(lib().fate_moe_layer_decode_workspace(C.byref(desc), C.byref(b), C.byref(o)))
    return b.value, o.value


def fate_moe_layer_decode(desc, x, Wg, bias, Wg_next, bias_next, m, renorm, topk_ids, topk_w, pred_ids, pred_w,
                          pred_pop, counts, offsets, perm, inv_perm, expert_order, experts_dev, shared_dev,
                          shared_gate, y, workspace, stream=None, hint_ids=None):
    out = fate_route_out(*[None if t is None else t.data_ptr() for t in
                           (topk_ids, topk_w, pred_ids, pred_w, pred_pop, counts, offsets, perm, inv_perm,
                            expert_order)])
    _check(lib().fate_moe_layer_decode(_stream(stream), C.byref(desc), _p(x), _p(Wg), _p(bias), _p(Wg_next),
                                       _p(bias_next), int(m), int(bool(renorm)), _p(hint_ids), C.byref(out), _p(experts_dev),
                                       _p(shared_dev), _p(shared_gate), _p(y), _p(workspace),
                                       C.c_size_t(workspace.numel() * workspace.element_size())))


def fate_moe_layer_decode_noalloc(desc, x, Wg, bias, Wg_next, bias_next, m, renorm, topk_ids, topk_w, pred_ids,
                                  pred_w, pred_pop, counts, offsets, perm, inv_perm, expert_order, experts_dev,
                                  shared_dev, shared_gate, y, status_dev, stream=None, hint_ids=None):
    out = fate_route_out(*[None if t is None else t.data_ptr() for t in
                           (topk_ids, topk_w, pred_ids, pred_w, pred_pop, counts, offsets, perm, inv_perm,
                            expert_order)])
    _check(lib().fate_moe_layer_decode_noalloc(_stream(stream), C.byref(desc), _p(x), _p(Wg), _p(bias),
                                               _p(Wg_next), _p(bias_next), int(m), int(bool(renorm)),
                                               _p(hint_ids), C.byref(out), _p(experts_dev), _p(shared_dev), _p(shared_gate),
                                               _p(y), _p(status_dev)))


def fate_profile_ffn_mfma_phase(desc, phase, x, experts_dev, counts, offsets, perm, inv_perm, expert_order, topk_w,
                                shared_dev, shared_gate, y, workspace, stream=None):
    _check(lib().fate_profile_ffn_mfma_phase(_stream(stream), C.byref(desc), int(phase), _p(x), _p(experts_dev),
                                             _p(counts), _p(offsets), _p(perm), _p(inv_perm), _p(expert_order),
                                             _p(topk_w), _p(shared_dev), _p(shared_gate), _p(y), _p(workspace),
                                             C.c_size_t(workspace.numel() * workspace.element_size())))


def fate_moe_ffn_q_workspace(desc):
    b = C.c_size_t(0)
    _check(lib().fate_moe_ffn_q_workspace(C.byref(desc), C.byref(b)))
    return b.value


def fate_moe_ffn_q(desc, x, experts_dev, counts, offsets, perm, inv_perm, expert_order, topk_w, shared_dev,
                   shared_gate, y, workspace, stream=None):
    _check(lib().fate_moe_ffn_q(_stream(stream), C.byref(desc), _p(x), _p(experts_dev), _p(counts), _p(offsets),
                                _p(perm), _p(inv_perm), _p(expert_order), _p(topk_w), _p(shared_dev), _p(shared_gate), _p(y),
                                _p(workspace), C.c_size_t(workspace.numel() * workspace.element_size())))


def fate_moe_ffn_q_part(desc, x, experts_dev, counts, offsets, perm, inv_perm, expert_order, topk_w, shared_dev,
                        shared_gate, y, workspace, part_experts, first, last, stream=None):
    arr = (C.c_int32 * max(1, len(part_experts)))(*part_experts)
    _check(lib().fate_moe_ffn_q_part(_stream(stream), C.byref(desc), _p(x), _p(experts_dev), _p(counts), _p(offsets),
                                     _p(perm), _p(inv_perm), _p(expert_order), _p(topk_w), _p(shared_dev),
                                     _p(shared_gate), _p(y), _p(workspace),
                                     C.c_size_t(workspace.numel() * workspace.element_size()), arr,
                                     len(part_experts), (1 if first else 0) | (2 if last else 0)))


# ---------------------------------------------------------------------------
# data preparation helpers (no arithmetic of the method: layout + pointer tables)
# ---------------------------------------------------------------------------


def fate_pack_scales(canonical, rows, groups, packed, stream=None):
    _check(lib().fate_pack_scales(_stream(stream), _p(canonical), rows, groups, _p(packed)))


class PackedExpert:
    """Device-native copy of one expert: packed codes + scales, kept alive."""

    def __init__(self, ex, device="cuda"):
        self.bits, self.group, self.I, self.H = ex.bits, ex.group, ex.I, ex.H
        self.t = {}
        for name, rows, K in (("w1", ex.I, ex.H), ("w3", ex.I, ex.H), ("w2", ex.H, ex.I)):
            src = getattr(ex, name).to(device).contiguous()
            dst = torch.empty_like(src)
            fate_pack_weight(src, rows, K, ex.bits, dst)
            self.t[name] = dst
        names = [("s1", ex.I, ex.H), ("s3", ex.I, ex.H), ("s2", ex.H, ex.I)]
        self.has_zero = getattr(ex, "z1", None) is not None
        if self.has_zero:                       # zero-points travel like scales (fp16 per group, group-major)
            names += [("z1", ex.I, ex.H), ("z3", ex.I, ex.H), ("z2", ex.H, ex.I)]
        for name, rows, K in names:
            src = getattr(ex, name).to(device).contiguous()
            dst = torch.empty_like(src).view(K // ex.group, rows)
            fate_pack_scales(src, rows, K // ex.group, dst)
            self.t[name] = dst
        torch.cuda.current_stream().synchronize()

    def struct(self):
        t = self.t
        z = [t[n].data_ptr() for n in ("z1", "z3", "z2")] if self.has_zero else [None, None, None]
        return fate_qexpert(t["w1"].data_ptr(), t["w3"].data_ptr(), t["w2"].data_ptr(), t["s1"].data_ptr(),
                            t["s3"].data_ptr(), t["s2"].data_ptr(), self.bits, self.group, self.I, 0, *z, 0)

    def nbytes(self):
        return sum(v.numel() * v.element_size() for v in self.t.values())


def expert_table(structs, device="cuda"):
    """Host list of fate_qexpert -> device array (uint8 tensor holding the structs)."""
    n = len(structs)
    arr = (fate_qexpert * max(n, 1))(*structs)
    raw = bytes(arr)[: n * C.sizeof(fate_qexpert)] if n else b""
    host = torch.frombuffer(bytearray(raw + b"\0" * 16), dtype=torch.uint8)
    return host.to(device)


def make_ffn_desc(N, H, E, k, I_max, bits, group, n_shared=0, I_shared_max=0, shared_bits=4, shared_group=128,
                  y_is_fp32=True, mode=0):
    return fate_ffn_desc(N, H, E, k, I_max, bits, group, n_shared, I_shared_max, shared_bits, shared_group,
                         int(y_is_fp32), mode, 0)
