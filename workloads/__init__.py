"""Seeded synthetic inputs for the MoE hot path.

This module produces tensors only: hidden states, gate matrices and biases,
and expert weights already in their stored (quantized) form.  It holds none
of the routing, permutation, dequantisation or FFN arithmetic; the CPU oracle
and the HIP library both receive what is generated here as plain data.
"""
from .configs import MoEShape, SHAPES, default_m  # noqa: F401
from .gen import (  # noqa: F401
    gen_hidden, gen_gate, gen_expert, gen_shared_gate, quantize_sym,
    QExpertHost, chain_next_hidden, unit_rmsnorm_bf16, gen_expert_unquantized,
)
