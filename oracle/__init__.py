"""CPU oracle of the MoE hot path (routing, cross-layer prediction,
permutation, dequantisation, SwiGLU FFN, expert-cache step).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of bench.py.  The library never calls into it, and nothing
here imports the library.
"""
