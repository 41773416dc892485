"""GPU parity of weight packing and of the quantised expert FFN against the
fp64 oracle, through the C ABI.  Bar: per token row
max_i |y_gpu - y_ref| / max_i |y_ref| <= 2e-3."""
import numpy as np
import pytest
import torch

from oracle import moe as O
import paper_2502_12224_amd.binding as B
from workloads import SHAPES, gen_gate, gen_hidden, quantize_sym
from helpers import DEV, GpuLayer, bias_np, f32, ffn_rel_err, gpu_permute, gpu_route, oracle_expert

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _expected_tiles(codes, rows, K, bits):
    """The documented device-native layout, written out independently with numpy."""
    q = O.unpack_codes(codes, bits)
    if bits == 4:
        u = (q + 8).astype(np.uint32)
        KT = 64
        out = np.zeros((rows // 32, K // KT, 64, 4), dtype=np.uint32)
        for half in range(2):
            for d in range(4):
                k0 = half * 32 + 8 * d
                blk = u.reshape(rows // 32, 32, K // KT, KT)[:, :, :, k0:k0 + 8]      # rb, n, kb, 8
                word = np.zeros(blk.shape[:3], dtype=np.uint32)
                for i in range(4):
                    word |= blk[..., 2 * i] << (4 * i)
                    word |= blk[..., 2 * i + 1] << (4 * i + 16)
                out[:, :, half * 32:(half + 1) * 32, d] = word.transpose(0, 2, 1)
        return out.reshape(-1)
    u = (q + 128).astype(np.uint8)
    KT = 32
    out = np.zeros((rows // 32, K // KT, 64, 16), dtype=np.uint8)
    blk = u.reshape(rows // 32, 32, K // KT, KT)
    for half in range(2):
        out[:, :, half * 32:(half + 1) * 32, :] = blk[:, :, :, half * 16:(half + 1) * 16].transpose(0, 2, 1, 3)
    return out.reshape(-1).view(np.uint32)


@pytest.mark.parametrize("bits,rows,K", [(4, 32, 64), (4, 96, 256), (8, 64, 128), (4, 1408, 2048), (8, 512, 256)])
def test_pack_weight_layout(bits, rows, K):
    g = torch.Generator().manual_seed(rows + K)
    w = torch.randn(rows, K, generator=g) * 0.02
    codes, _ = quantize_sym(w, bits, 64)
    src = codes.to(DEV)
    dst = torch.zeros_like(src)
    B.fate_pack_weight(src, rows, K, bits, dst)
    torch.cuda.synchronize()
    got = dst.cpu().numpy().reshape(-1).view(np.uint32)
    assert np.array_equal(got, _expected_tiles(codes.numpy(), rows, K, bits))


def _layer_case(name, N, layer=0, mode=0, y_is_fp32=True, seed_step=0):
    cfg = SHAPES[name]
    x = gen_hidden(cfg, N, step=seed_step, device=DEV)
    Wg, b = gen_gate(cfg, layer, device=DEV)
    ids, w, _ = gpu_route(x, Wg, b, cfg.k, cfg.renorm, want_probs=False)
    counts, offsets, perm, inv, order = gpu_permute(ids, cfg.E)
    torch.cuda.synchronize()
    used = sorted(set(ids.cpu().numpy().ravel().tolist()))
    L = GpuLayer(cfg, layer, experts=used)
    y, ws = L.ffn(x, counts, offsets, perm, inv, order, w, mode=mode, y_is_fp32=y_is_fp32)
    assert int(ws[:4].view(torch.int32)[0]) == 0
    # the oracle gets the same x, the GPU's routing (checked elsewhere) and the same stored weights
    experts = {e: oracle_expert(L.host[e]) for e in used}
    shared = [oracle_expert(ex) for ex in L.shared_host]
    sg = None if L.shared_gate is None else f32(L.shared_gate)
    y_ref = O.moe_ffn(f32(x), ids.cpu().numpy(), w.cpu().numpy().astype(np.float64), experts, shared, sg)
    return f32(y), y_ref


@pytest.mark.parametrize("name,N", [("tiny", 1), ("tiny", 16), ("qwen", 1), ("qwen", 5), ("deepseek", 8),
                                    ("deepseek", 13), ("mixtral", 1), ("mixtral", 3)])
def test_ffn_decode_matches_oracle(name, N):
    y, y_ref = _layer_case(name, N, mode=1)
    err = ffn_rel_err(y, y_ref)
    assert np.isfinite(y).all()
    assert err.max() <= TOL, err


def test_ffn_decode_bf16_output():
    y, y_ref = _layer_case("tiny", 7, mode=1, y_is_fp32=False)
    err = ffn_rel_err(y, y_ref)
    assert err.max() <= 2 ** -8 + TOL          # one bf16 rounding of the result on top


def test_ffn_flags_missing_expert():
    cfg = SHAPES["tiny"]
    N = 4
    x = gen_hidden(cfg, N, device=DEV)
    Wg, b = gen_gate(cfg, 0, device=DEV)
    ids, w, _ = gpu_route(x, Wg, b, cfg.k, cfg.renorm, want_probs=False)
    counts, offsets, perm, inv, order = gpu_permute(ids, cfg.E)
    used = sorted(set(ids.cpu().numpy().ravel().tolist()))
    L = GpuLayer(cfg, 0, experts=used[1:])        # one activated expert is not on the device
    y, ws = L.ffn(x, counts, offsets, perm, inv, order, w, mode=1)
    assert int(ws[:4].view(torch.int32)[0]) != 0
    # the missing expert's pairs contribute nothing, everything else is as usual
    ids_h = ids.cpu().numpy()
    w_ref = w.cpu().numpy().astype(np.float64)
    w_ref[ids_h == used[0]] = 0.0
    experts = {e: oracle_expert(L.host[e]) for e in used[1:]}
    experts[used[0]] = experts[used[1]]          # (weight 0: any expert will do)
    y_ref = O.moe_ffn(f32(x), ids_h, w_ref, experts, [oracle_expert(ex) for ex in L.shared_host],
                      None if L.shared_gate is None else f32(L.shared_gate))
    assert ffn_rel_err(f32(y), y_ref).max() <= TOL


@pytest.mark.parametrize("name,N", [("qwen", 5), ("deepseek", 13), ("mixtral", 3), ("tiny", 16)])
def test_ffn_decode_is_reproducible_bit_for_bit(name, N):
    """The decode kernels store partial outputs and add them in a fixed order: two runs on the same inputs (the
    second one over a workspace filled with other values) give the same bits."""
    cfg = SHAPES[name]
    x = gen_hidden(cfg, N, device=DEV)
    Wg, b = gen_gate(cfg, 0, device=DEV)
    ids, w, _ = gpu_route(x, Wg, b, cfg.k, cfg.renorm, want_probs=False)
    counts, offsets, perm, inv, order = gpu_permute(ids, cfg.E)
    torch.cuda.synchronize()
    used = sorted(set(ids.cpu().numpy().ravel().tolist()))
    L = GpuLayer(cfg, 0, experts=used)
    y1, ws = L.ffn(x, counts, offsets, perm, inv, order, w, mode=1)
    y1 = y1.clone()
    outs = []
    for rep in range(3):
        y2, ws2 = L.ffn(x, counts, offsets, perm, inv, order, w, mode=1, ws_fill=0x7f if rep else 0)
        assert int(ws2[:4].view(torch.int32)[0]) == 0
        outs.append(y2.clone())
    for y2 in outs:
        assert torch.equal(y1, y2)


def _mfma_case(name, N, rows=None, layer=0, y_is_fp32=True):
    """MFMA path on N tokens; oracle on `rows` (all rows if None)."""
    cfg = SHAPES[name]
    x = gen_hidden(cfg, N, device=DEV)
    Wg, b = gen_gate(cfg, layer, device=DEV)
    ids, w, _ = gpu_route(x, Wg, b, cfg.k, cfg.renorm, want_probs=False)
    counts, offsets, perm, inv, order = gpu_permute(ids, cfg.E)
    torch.cuda.synchronize()
    used = sorted(set(ids.cpu().numpy().ravel().tolist()))
    L = GpuLayer(cfg, layer, experts=used)
    y, ws = L.ffn(x, counts, offsets, perm, inv, order, w, mode=2, y_is_fp32=y_is_fp32)
    assert int(ws[:4].view(torch.int32)[0]) == 0
    rows = list(range(N)) if rows is None else rows
    ids_h = ids.cpu().numpy()
    need = sorted(set(ids_h[rows].ravel().tolist()))
    experts = {e: oracle_expert(L.host[e]) for e in need}
    shared = [oracle_expert(ex) for ex in L.shared_host]
    sg = None if L.shared_gate is None else f32(L.shared_gate)
    y_ref = O.moe_ffn_rows(f32(x), ids_h, w.cpu().numpy().astype(np.float64), experts, shared, sg, rows=rows)
    yg = f32(y)
    assert np.isfinite(yg).all()
    return yg[rows], y_ref, counts.cpu().numpy()


@pytest.mark.parametrize("name,N,rows", [
    ("tiny", 16, None), ("tiny", 200, None), ("tiny", 1, None), ("tiny", 129, None),
    ("qwen_prefill", 48, [0, 7, 47]), ("deepseek", 40, [1, 20, 39]), ("mixtral", 20, [3, 11]),
])
def test_ffn_mfma_matches_oracle(name, N, rows):
    y, y_ref, counts = _mfma_case(name, N, rows)
    err = ffn_rel_err(y, y_ref)
    print(f"{name} N={N}: max row err {err.max():.2e}, busiest expert {counts.max()} rows")
    assert err.max() <= TOL, err


def test_ffn_mfma_bf16_output():
    y, y_ref, _ = _mfma_case("tiny", 70, None, y_is_fp32=False)
    assert ffn_rel_err(y, y_ref).max() <= 2 ** -8 + TOL


@pytest.mark.parametrize("name,N,rows", [
    ("qwen_prefill", 2048, [0, 511, 1024, 2047]),     # Zipf-skewed routing
    ("qwen_prefill", 512, [3, 256, 511]),
    ("deepseek", 1024, [0, 500, 1023]),               # two int8 shared experts beside the int4 routed ones
    ("mixtral", 2048, [5, 2047]),                     # 90.8 MB experts, I = 14336
])
def test_ffn_mfma_full_size_sampled_rows(name, N, rows):
    """The prefill sizes the bench times, in its launch configuration (auto
    mode picks the MFMA path); oracle on sampled token rows."""
    cfg = SHAPES[name]
    y, y_ref, counts = _mfma_case(name, N, rows)
    err = ffn_rel_err(y, y_ref)
    print(f"{name} N={N}: max row err {err.max():.2e}; expert rows min/max {counts.min()}/{counts.max()}")
    assert counts.sum() == N * cfg.k and err.max() <= TOL, err
