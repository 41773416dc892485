"""Shapes of the five synthetic MoE workloads.

Each entry mirrors one of the benchmark configurations: a tiny 2-layer case,
a Qwen1.5-MoE-shaped stack (60 fine-grained experts + one gated shared
expert), a DeepSeek-MoE-16B-shaped stack (64 experts + 2 shared) and a
Mixtral-8x7B-shaped stack (8 large experts).  The two model families are the
ones the paper evaluates (section 5.1, "Models"); Mixtral is the conventional
top-k design of its figure 2(a).
"""
from dataclasses import dataclass, field
from typing import Optional


@dataclass(frozen=True)
class MoEShape:
    name: str
    layers: int
    H: int                 # hidden size
    E: int                 # routed experts per layer
    k: int                 # experts per token
    I: int                 # routed expert intermediate size
    bits: int              # routed expert code width (4 or 8)
    group: int             # quantisation group along the reduction dim
    n_shared: int = 0
    I_shared: int = 0
    shared_bits: int = 4
    shared_gate: bool = False      # sigmoid(x . w_sg) on the shared expert
    renorm: bool = False           # renormalise top-k weights to sum to 1
    gate_var: float = 0.0          # variance of gate weights (std = sqrt)
    bias_std: float = 0.0          # N(0, bias_std) per-expert gate bias
    zipf_s: float = 0.0            # >0: bias = -s*ln(rank) under a seeded permutation
    w_std: float = 0.02            # expert weight std before quantisation
    seed: int = 0
    cache_frac: float = 1.0        # fraction of routed experts resident on device
    L_shallow: int = 3             # number of fully cached shallow layers

    @property
    def m(self) -> int:
        return default_m(self.E, self.k)


def default_m(E: int, k: int) -> int:
    """Width of the widened prefetch set: experts strictly above the 75th
    percentile (linear interpolation) of one token's E routing weights."""
    m = E - 1 - (3 * (E - 1)) // 4
    return max(k, min(E, m))


SHAPES = {
    # configs[0]
    "tiny": MoEShape("tiny", layers=2, H=256, E=8, k=2, I=512, bits=8, group=64,
                     renorm=True, gate_var=1.0 / 256, seed=0),
    # configs[1] / configs[2]
    "qwen": MoEShape("qwen", layers=24, H=2048, E=60, k=4, I=1408, bits=4, group=128,
                     n_shared=1, I_shared=5632, shared_bits=4, shared_gate=True,
                     renorm=False, gate_var=1.0 / 2048, bias_std=0.5, seed=1),
    "qwen_prefill": MoEShape("qwen_prefill", layers=24, H=2048, E=60, k=4, I=1408, bits=4, group=128,
                             n_shared=1, I_shared=5632, shared_bits=4, shared_gate=True,
                             renorm=False, gate_var=1.0 / 2048, zipf_s=1.1, seed=2),
    # configs[3]
    "deepseek": MoEShape("deepseek", layers=28, H=2048, E=64, k=6, I=1408, bits=4, group=128,
                         n_shared=2, I_shared=1408, shared_bits=8, shared_gate=False,
                         renorm=False, gate_var=1.0 / 2048, seed=3, cache_frac=0.30),
    # configs[4]
    "mixtral": MoEShape("mixtral", layers=32, H=4096, E=8, k=2, I=14336, bits=4, group=128,
                        renorm=True, gate_var=1.0 / 4096, seed=4, cache_frac=0.25),
}
