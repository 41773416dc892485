"""Seeded tensor generators (torch; any device).

Everything here is input preparation.  Expert weights are drawn in fp32 and
stored in the symmetric group-quantised form the benchmark configurations
name (int8 / int4 codes plus one fp16 scale per group of consecutive elements
along the reduction dimension of an output row); what the hot path receives
are those codes and scales.  The storage format ("canonical layout"):

  int8: one two's-complement byte per code, row-major [rows, K].
  int4: unsigned nibble u = q + 8, two per byte, low nibble = even column,
        row-major [rows, K/2].
  int2: field u in 0..3 (level (2u - 3) * scale), four per byte, column 4b+i in bits 2i..2i+1
        of byte b, row-major [rows, K/4].
  scales: fp16, row-major [rows, K/group].
"""
from dataclasses import dataclass
from typing import Optional
import math
import torch

from .configs import MoEShape

_KIND = {"hidden": 1, "gate": 2, "bias": 3, "expert": 4, "shared": 5, "sgate": 6, "perm": 7}


def _gen(device, *key: int) -> torch.Generator:
    # 64-bit mix of the key tuple (splitmix-style); only decides the stream.
    s = 0x9E3779B97F4A7C15
    for v in key:
        s = (s ^ (int(v) + 0x9E3779B97F4A7C15 + ((s << 6) & 0xFFFFFFFFFFFFFFFF) + (s >> 2))) & 0xFFFFFFFFFFFFFFFF
        s = (s * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        s ^= s >> 31
    g = torch.Generator(device=device)
    g.manual_seed(s & 0x7FFFFFFFFFFFFFFF)
    return g


def gen_hidden(cfg: MoEShape, N: int, step: int = 0, device="cpu") -> torch.Tensor:
    """Gate input of the first layer: N(0,1) in fp32, cast to bf16.  [N, H]."""
    g = _gen(device, cfg.seed, _KIND["hidden"], step, N)
    return torch.randn(N, cfg.H, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)


def gen_gate(cfg: MoEShape, layer: int, device="cpu"):
    """Gate matrix [E, H] bf16 (variance gate_var) and bias [E] fp32 or None."""
    g = _gen(device, cfg.seed, _KIND["gate"], layer)
    Wg = (torch.randn(cfg.E, cfg.H, generator=g, device=device, dtype=torch.float32)
          * math.sqrt(cfg.gate_var)).to(torch.bfloat16)
    bias = None
    if cfg.zipf_s > 0:
        gp = _gen("cpu", cfg.seed, _KIND["perm"], layer)
        pi = torch.randperm(cfg.E, generator=gp)
        ranks = torch.arange(1, cfg.E + 1, dtype=torch.float64)
        b = torch.empty(cfg.E, dtype=torch.float64)
        b[pi] = -cfg.zipf_s * torch.log(ranks)
        bias = b.to(torch.float32).to(device)
    elif cfg.bias_std > 0:
        gb = _gen(device, cfg.seed, _KIND["bias"], layer)
        bias = torch.randn(cfg.E, generator=gb, device=device, dtype=torch.float32) * cfg.bias_std
    return Wg, bias


def gen_shared_gate(cfg: MoEShape, layer: int, device="cpu") -> Optional[torch.Tensor]:
    """Shared-expert gate vector [H] bf16 (variance 1/H), or None."""
    if not cfg.shared_gate:
        return None
    g = _gen(device, cfg.seed, _KIND["sgate"], layer)
    return (torch.randn(cfg.H, generator=g, device=device, dtype=torch.float32)
            / math.sqrt(cfg.H)).to(torch.bfloat16)


def quantize_sym(w: torch.Tensor, bits: int, group: int):
    """Symmetric group quantiser used to prepare stored weights.

    w: [rows, K] fp32.  Returns (codes uint8 canonical layout, scales fp16).
    scale = fp16(max|w| / qmax) per group (1 for an all-zero group), code =
    round-half-even(w / scale) clamped to [-qmax, qmax].
    """
    assert bits in (2, 4, 8)
    rows, K = w.shape
    assert K % group == 0 and group % 4 == 0
    if bits == 2:
        # four levels -3s, -s, s, 3s with s = fp16(max|w| / 3) (0 for an all-zero group); field u = (q + 3) / 2
        wg = w.reshape(rows, K // group, group)
        s = (wg.abs().amax(dim=-1) / 3).to(torch.float16)
        sf = s.to(torch.float32).unsqueeze(-1)
        u = torch.where(sf > 0, torch.round((wg / torch.where(sf > 0, sf, torch.ones_like(sf)) + 3) / 2),
                        torch.zeros_like(wg))
        u = torch.clamp(u, 0, 3).reshape(rows, K).to(torch.uint8)
        codes = u[:, 0::4] | (u[:, 1::4] << 2) | (u[:, 2::4] << 4) | (u[:, 3::4] << 6)
        return codes.contiguous(), s.contiguous()
    qmax = 127 if bits == 8 else 7
    wg = w.reshape(rows, K // group, group)
    s = (wg.abs().amax(dim=-1) / qmax).to(torch.float16)
    s = torch.where(s == 0, torch.ones_like(s), s)
    q = torch.clamp(torch.round(wg / s.to(torch.float32).unsqueeze(-1)), -qmax, qmax)
    q = q.reshape(rows, K).to(torch.int16)
    if bits == 8:
        codes = q.to(torch.int8).view(torch.uint8)
    else:
        u = (q + 8).to(torch.uint8)
        codes = u[:, 0::2] | (u[:, 1::2] << 4)
    return codes.contiguous(), s.contiguous()


def quantize_minmax(w: torch.Tensor, bits: int, group: int):
    """Asymmetric group quantiser (plain min / max) used to prepare stored weights with zero-points.

    w: [rows, K] fp32.  Returns (fields uint8 canonical layout, scales fp16, zero-points fp16):
    w ~ (u - z) * s with u in [0, 2^bits - 1], s = fp16((max - min) / (2^bits - 1)) per group
    (1 for a constant group), z = fp16(-min / s), u = round-half-even(w / s + z) clamped.
    """
    assert bits in (2, 4)
    rows, K = w.shape
    assert K % group == 0 and group % 4 == 0
    umax = (1 << bits) - 1
    wg = w.reshape(rows, K // group, group)
    lo, hi = wg.amin(dim=-1), wg.amax(dim=-1)
    s = ((hi - lo) / umax).to(torch.float16)
    s = torch.where(s == 0, torch.ones_like(s), s)
    sf = s.to(torch.float32)
    z = (-lo / sf).to(torch.float16)
    u = torch.clamp(torch.round(wg / sf.unsqueeze(-1) + z.to(torch.float32).unsqueeze(-1)), 0, umax)
    u = u.reshape(rows, K).to(torch.uint8)
    if bits == 4:
        codes = u[:, 0::2] | (u[:, 1::2] << 4)
    else:
        codes = u[:, 0::4] | (u[:, 1::4] << 2) | (u[:, 2::4] << 4) | (u[:, 3::4] << 6)
    return codes.contiguous(), s.contiguous(), z.contiguous()


@dataclass
class QExpertHost:
    """One SwiGLU expert in canonical stored form (torch tensors, any device)."""
    w1: torch.Tensor  # gate proj   [I, H] codes
    w3: torch.Tensor  # up proj     [I, H] codes
    w2: torch.Tensor  # down proj   [H, I] codes
    s1: torch.Tensor
    s3: torch.Tensor
    s2: torch.Tensor
    bits: int
    group: int
    I: int
    H: int
    z1: Optional[torch.Tensor] = None   # zero-points (formats that have them), shaped like the scales
    z3: Optional[torch.Tensor] = None
    z2: Optional[torch.Tensor] = None

    def _tensors(self):
        return [t for t in (self.w1, self.w3, self.w2, self.s1, self.s3, self.s2, self.z1, self.z3, self.z2)
                if t is not None]

    def nbytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in self._tensors())

    def cpu(self) -> "QExpertHost":
        c = lambda t: None if t is None else t.cpu()
        return QExpertHost(self.w1.cpu(), self.w3.cpu(), self.w2.cpu(), self.s1.cpu(), self.s3.cpu(),
                           self.s2.cpu(), self.bits, self.group, self.I, self.H, c(self.z1), c(self.z3), c(self.z2))


def gen_expert(cfg: MoEShape, layer: int, e: int, shared: bool = False, device="cpu", bits: Optional[int] = None,
               group: Optional[int] = None, zero_points: bool = False) -> QExpertHost:
    """Expert e of a layer: three N(0, w_std) matrices, quantised.  bits / group override the
    configuration's format: the same weights (same random stream) stored at another width;
    zero_points stores them in the asymmetric format (4 or 2 bits)."""
    I = cfg.I_shared if shared else cfg.I
    bits = bits or (cfg.shared_bits if shared else cfg.bits)
    group = group or cfg.group
    g = _gen(device, cfg.seed, _KIND["shared" if shared else "expert"], layer, e)
    mats = []
    for rows, K in ((I, cfg.H), (I, cfg.H), (cfg.H, I)):
        w = torch.randn(rows, K, generator=g, device=device, dtype=torch.float32) * cfg.w_std
        mats.append(quantize_minmax(w, bits, group) if zero_points else quantize_sym(w, bits, group))
        del w
    if zero_points:
        (w1, s1, z1), (w3, s3, z3), (w2, s2, z2) = mats
        return QExpertHost(w1, w3, w2, s1, s3, s2, bits, group, I, cfg.H, z1, z3, z2)
    (w1, s1), (w3, s3), (w2, s2) = mats
    return QExpertHost(w1, w3, w2, s1, s3, s2, bits, group, I, cfg.H)


def gen_expert_unquantized(cfg: MoEShape, layer: int, e: int, shared: bool = False, device="cpu"):
    """The fp32 matrices (W1, W3, W2) that gen_expert quantises: reference for the reported
    quantisation error of a stored format."""
    I = cfg.I_shared if shared else cfg.I
    g = _gen(device, cfg.seed, _KIND["shared" if shared else "expert"], layer, e)
    return tuple(torch.randn(rows, K, generator=g, device=device, dtype=torch.float32) * cfg.w_std
                 for rows, K in ((I, cfg.H), (I, cfg.H), (cfg.H, I)))


def unit_rmsnorm_bf16(h: torch.Tensor) -> torch.Tensor:
    """Harness glue for a chained stack: x = bf16(h / rms(h)) per row."""
    h = h.to(torch.float32)
    return (h * torch.rsqrt((h * h).mean(dim=-1, keepdim=True))).to(torch.bfloat16)


def chain_next_hidden(h: torch.Tensor, y: torch.Tensor) -> torch.Tensor:
    """Harness glue: residual stream h_{l+1} = h_l + y_l (fp32)."""
    return h.to(torch.float32) + y.to(torch.float32)
