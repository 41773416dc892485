"""Full-size parity in the launch configuration bench.py times: the
Qwen1.5-MoE-shaped decode layer (batch 1, fused routing, decode FFN kernels)
driven through the stack harness, teacher-forced against the oracle."""
import numpy as np
import pytest
import torch

from oracle import moe as O
from paper_2502_12224_amd.stack import LayerBuffers, MoEStack, layer_forward
from workloads import SHAPES, gen_expert, gen_hidden, unit_rmsnorm_bf16, chain_next_hidden
from helpers import DEV, bias_np, f32, ffn_rel_err, oracle_expert

pytestmark = pytest.mark.gpu


def test_qwen_decode_layers_match_oracle_teacher_forced():
    cfg = SHAPES["qwen"]
    stack = MoEStack(cfg, DEV, layers=3)
    buf = LayerBuffers(cfg, 1, DEV)
    assert buf.fused_ok
    worst = 0.0
    for step in range(2):
        h = gen_hidden(cfg, 1, step=step, device=DEV).float()
        for l in range(2):
            x = unit_rmsnorm_bf16(h)
            y = layer_forward(cfg, stack.layers[l], stack.layers[l + 1], x, buf)
            torch.cuda.synchronize()
            lw, ln = stack.layers[l], stack.layers[l + 1]
            rid, rw, _, rz = O.gate_route(f32(x), f32(lw.Wg), bias_np(lw.bias), cfg.k, cfg.renorm)
            pid, _, pop, pz = O.cross_layer_predict(f32(x), f32(ln.Wg), bias_np(ln.bias), cfg.m)
            assert len(O.near_tie_rows(rz, cfg.k)) == 0 and len(O.near_tie_rows(pz, cfg.m)) == 0
            assert np.array_equal(buf.ids.cpu().numpy(), rid)
            assert np.array_equal(buf.pred_ids.cpu().numpy(), pid)
            assert np.array_equal(buf.pred_pop.cpu().numpy(), pop)
            ref = O.permute(rid, cfg.E)
            for a, r in zip((buf.counts, buf.offsets, buf.perm[:cfg.k], buf.inv_perm[:cfg.k], buf.order), ref):
                assert np.array_equal(a.cpu().numpy(), r)
            assert np.abs(buf.w.cpu().numpy() - rw).max() <= 1e-6
            experts = {int(e): oracle_expert(gen_expert(cfg, l, int(e), device=DEV)) for e in rid.ravel()}
            shared = [oracle_expert(gen_expert(cfg, l, 0, shared=True, device=DEV))]
            y_ref = O.moe_ffn(f32(x), rid, rw, experts, shared, f32(lw.shared_gate))
            err = ffn_rel_err(f32(y), y_ref).max()
            worst = max(worst, err)
            assert err <= 2e-3, (step, l, err)
            h = chain_next_hidden(h, y)
    print(f"worst FFN row error {worst:.2e}")
