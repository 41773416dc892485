"""The decode layer call that allocates nothing (its workspace is a device
array built into the library) against the call with a caller-owned workspace:
same kernels, so every output must be equal bit for bit; two calls in a row,
the second on a smaller input."""
import numpy as np
import pytest
import torch

import paper_2502_12224_amd.binding as B
from paper_2502_12224_amd.stack import LayerBuffers, LayerWeights, layer_forward
from workloads import SHAPES, gen_hidden
from helpers import DEV

pytestmark = pytest.mark.gpu

FIELDS = ("ids", "w", "pred_ids", "pred_w", "pred_pop", "counts", "offsets", "perm", "inv_perm", "order", "y")


def _noalloc(cfg, lw, ln, x, buf, status):
    B.fate_moe_layer_decode_noalloc(buf.desc, x, lw.Wg, lw.bias, ln.Wg, ln.bias, cfg.m, cfg.renorm, buf.ids, buf.w,
                                    buf.pred_ids, buf.pred_w, buf.pred_pop, buf.counts, buf.offsets, buf.perm,
                                    buf.inv_perm, buf.order, lw.table, lw.shared_table, lw.shared_gate, buf.y,
                                    status)


def test_no_alloc_layer_call_equals_the_workspace_call():
    cfg = SHAPES["qwen"]
    lw = LayerWeights(cfg, 0, DEV)
    ln = LayerWeights(cfg, 1, DEV, experts=[])
    status = torch.zeros(4, dtype=torch.int32, device=DEV)
    for N in (4, 1):                       # the second call is smaller and finds the first one's leftovers
        print(f"no-alloc layer call, N = {N}", flush=True)
        x = gen_hidden(cfg, N, step=N, device=DEV)
        ref, got = LayerBuffers(cfg, N, DEV), LayerBuffers(cfg, N, DEV)
        layer_forward(cfg, lw, ln, x, ref, one_launch=True)
        torch.cuda.synchronize()
        assert ref.status() == 0
        got.y.fill_(float("nan"))
        _noalloc(cfg, lw, ln, x, got, status)
        torch.cuda.synchronize()
        assert int(status[0]) == 0
        for f in FIELDS:
            assert torch.equal(getattr(got, f), getattr(ref, f)), (f, N)
        assert np.isfinite(got.y.cpu().numpy()).all()


def test_no_alloc_layer_call_rejects_shapes_beyond_its_scratch():
    cfg = SHAPES["mixtral"]
    N = 4                                  # 4 tokens x 2 experts x 448 blocks x 16 KiB rows > 32 MiB
    buf = LayerBuffers(cfg, N, DEV)
    nbytes, _ = B.fate_moe_layer_decode_workspace(buf.desc)
    assert nbytes > (32 << 20)
    p = torch.zeros(64, dtype=torch.uint8, device=DEV)      # never dereferenced: the size check comes first
    status = torch.zeros(4, dtype=torch.int32, device=DEV)
    with pytest.raises(B.FateError) as e:
        B.fate_moe_layer_decode_noalloc(buf.desc, p, p, None, None, None, cfg.m, cfg.renorm, buf.ids, buf.w, None,
                                        None, None, buf.counts, buf.offsets, buf.perm, buf.inv_perm, buf.order, p,
                                        None, None, buf.y, status)
    assert e.value.status == 4 and "scratch" in str(e.value)
