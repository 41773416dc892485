#!/usr/bin/env python3
"""Benchmark of the MoE hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

Workloads (all synthetic, seeded):
  qwen_decode (default)  Qwen1.5-MoE-shaped stack, 24 layers, batch 1 decode.
                         A step is one token through all 24 layers: fused
                         routing + cross-layer prediction + permutation, the
                         quantised expert FFN, and the cache step.
  qwen_prefill512 / qwen_prefill2048 / deepseek_prefill1024 / mixtral_prefill2048
                         one prefill pass of N tokens through the stack's layers.
  deepseek_offload / mixtral_offload
                         experts in pinned host memory, a fraction cached on the
                         device: one prefill pass, then decode steps with the cache
                         step issuing H2D copies on a side stream.
Prints one JSON line (see the design doc for the fields).
"""
import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_sources_id():
    """sha256 (first 16 hex digits) over the library's sources: names the build a stored counter figure belongs to."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2502_12224_amd", "csrc")
    for f in sorted(os.listdir(csrc)):
        if f.endswith((".hip", ".h", ".cpp")):
            h.update(f.encode())
            h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(name):
    """HBM bytes per launch from the counter runs summarised under profiles/.  The summary names the
    sources it was taken on (kernel_sources_id); a figure of another build is not reported (None)."""
    path = os.path.join(ROOT, "profiles", name)
    val = src = None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                val = float(line.split("=")[1])
            if line.startswith("kernel_sources_id"):
                src = line.split("=")[1].strip()
    except OSError:
        return None
    if val is None or src != kernel_sources_id():
        log(f"[bench] {name}: counters were taken on sources {src}, this build is {kernel_sources_id()} -> traffic null")
        return None
    return val


def blas_threads():
    """Threads the numpy oracle's matrix products really use (the BLAS pool), not the affinity mask."""
    try:
        from threadpoolctl import threadpool_info
        n = [p["num_threads"] for p in threadpool_info() if p.get("user_api") == "blas"]
        if n:
            return max(n)
    except Exception:
        pass
    return len(os.sched_getaffinity(0))


def expert_bytes(H, I, bits, group):
    """Algorithmic bytes of one expert: codes + fp16 scales of W1, W3, W2."""
    return 3 * (H * I * bits // 8 + H * I // group * 2)


def cpu_baseline_decode(cfg, xs, layers_sample, tokens_sample):
    """Times the plain fp64 oracle on host cores for a bounded sample."""
    import numpy as np
    import torch
    from oracle import moe as O
    from workloads import gen_expert, gen_gate, gen_shared_gate
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    dev = "cuda"
    # stage the stored weights of the sampled layers on the host first (not timed)
    staged = {}
    for l in sorted(set(layers_sample) | {l + 1 for l in layers_sample if l + 1 < cfg.layers}):
        Wg, b = gen_gate(cfg, l, dev)
        staged[l] = dict(Wg=Wg.float().cpu().numpy(), b=None if b is None else b.cpu().numpy(),
                         sg=gen_shared_gate(cfg, l, dev), experts={}, shared=[])
        if staged[l]["sg"] is not None:
            staged[l]["sg"] = staged[l]["sg"].float().cpu().numpy()
    t_total = 0.0
    n_units = 0
    for s in tokens_sample:
        for l in layers_sample:
            x = xs[s, l].float().cpu().numpy()
            st = staged[l]
            ids, w, _, _ = O.gate_route(x, st["Wg"], st["b"], cfg.k, cfg.renorm)
            need = sorted(set(ids.ravel().tolist()))
            host = {e: gen_expert(cfg, l, e, device=dev).cpu() for e in need}
            sh = [gen_expert(cfg, l, i, shared=True, device=dev).cpu() for i in range(cfg.n_shared)]
            t0 = time.perf_counter()
            ids, w, _, _ = O.gate_route(x, st["Wg"], st["b"], cfg.k, cfg.renorm)
            if l + 1 < cfg.layers and (l + 1) in staged:
                O.cross_layer_predict(x, staged[l + 1]["Wg"], staged[l + 1]["b"], cfg.m)
            O.permute(ids, cfg.E)
            ex = {e: O.OracleExpert(h.w1.numpy(), h.s1.numpy(), h.w3.numpy(), h.s3.numpy(), h.w2.numpy(),
                                    h.s2.numpy(), h.bits, h.group) for e, h in host.items()}
            shx = [O.OracleExpert(h.w1.numpy(), h.s1.numpy(), h.w3.numpy(), h.s3.numpy(), h.w2.numpy(),
                                  h.s2.numpy(), h.bits, h.group) for h in sh]
            O.moe_ffn(x, ids, w, ex, shx, st["sg"])
            t_total += time.perf_counter() - t0
            n_units += 1
    per_layer_token = t_total / n_units
    return per_layer_token, n_units, t_total


def cpu_baseline_prefill(cfg, x, layer, rows):
    """Oracle time for one layer: routing / prediction / permutation of all tokens, FFN of `rows`."""
    import torch
    from oracle import moe as O
    from workloads import gen_expert, gen_gate, gen_shared_gate
    dev = "cuda"
    Wg, b = gen_gate(cfg, layer, dev)
    Wg2, b2 = gen_gate(cfg, layer + 1, dev)
    sg = gen_shared_gate(cfg, layer, dev)
    xn = x.float().cpu().numpy()
    Wg, Wg2 = Wg.float().cpu().numpy(), Wg2.float().cpu().numpy()
    b = None if b is None else b.cpu().numpy()
    b2 = None if b2 is None else b2.cpu().numpy()
    sg = None if sg is None else sg.float().cpu().numpy()
    ids, w, _, _ = O.gate_route(xn, Wg, b, cfg.k, cfg.renorm)
    need = sorted(set(ids[rows].ravel().tolist()))
    host = {e: gen_expert(cfg, layer, e, device=dev).cpu() for e in need}
    sh = [gen_expert(cfg, layer, i, shared=True, device=dev).cpu() for i in range(cfg.n_shared)]
    mk = lambda h: O.OracleExpert(h.w1.numpy(), h.s1.numpy(), h.w3.numpy(), h.s3.numpy(), h.w2.numpy(),
                                  h.s2.numpy(), h.bits, h.group)
    t0 = time.perf_counter()
    ids, w, _, _ = O.gate_route(xn, Wg, b, cfg.k, cfg.renorm)
    O.cross_layer_predict(xn, Wg2, b2, cfg.m)
    O.permute(ids, cfg.E)
    t_route = time.perf_counter() - t0
    t0 = time.perf_counter()
    O.moe_ffn_rows(xn, ids, w, {e: mk(h) for e, h in host.items()}, [mk(h) for h in sh], sg, rows=rows)
    t_ffn = time.perf_counter() - t0
    return t_route, t_ffn


def bench_decode(args):
    import numpy as np
    import torch
    import paper_2502_12224_amd.binding as B
    from paper_2502_12224_amd.stack import LayerBuffers, MoEStack, layer_forward
    from workloads import SHAPES

    shape, N, S, desc = DECODE_WORKLOADS[args.workload]
    qwen = args.workload == "qwen_decode"
    cfg = SHAPES[shape]
    dev = "cuda"
    L, E, H = cfg.layers, cfg.E, cfg.H
    t0 = time.time()
    log(f"[bench] generating {L} layers x ({E} routed + {cfg.n_shared} shared) experts on the device ...")
    stack = MoEStack(cfg, dev, progress=lambda l: log(f"[bench]   layer {l} packed ({time.time() - t0:.0f}s)") if l % 6 == 5 else None)
    log(f"[bench] weights resident: {stack.nbytes() / 1e9:.2f} GB")

    # untimed free-running chain: the gate inputs of every layer and step
    xs, true_ids, pred_ids = stack.chain(N, S)
    torch.cuda.synchronize()
    log(f"[bench] chained {S} decode steps ({time.time() - t0:.0f}s)")
    t_ids = true_ids.cpu().numpy()       # [S, L, N, k]
    p_ids = pred_ids.cpu().numpy()       # [S, L, N, m]  (prediction made at layer l for layer l+1)
    # reporting (untimed): the oracle's definitions of the accuracy figures, the prediction made
    # at layer l against the true routing of layer l+1
    from oracle import moe as O
    acc = [O.prediction_accuracy(p_ids[s, l], t_ids[s, l + 1], cfg.k) for s in range(S) for l in range(L - 1)]
    acc_k = float(np.mean([v[0] for v in acc]))
    rec_m = float(np.mean([v[1] for v in acc]))
    # rows whose fp64 logits have a top-k gap below 1e-5 (their selection may legitimately differ from fp64)
    near_ties = 0
    for l in range(L):
        lw = stack.layers[l]
        z = O.gate_logits(xs[:, l].reshape(S * N, H).float().cpu().numpy(), lw.Wg.float().cpu().numpy(),
                          None if lw.bias is None else lw.bias.cpu().numpy())
        near_ties += len(O.near_tie_rows(z, cfg.k))

    # per-layer buffers whose counts / predicted popularity sit in one arena
    bufs = [LayerBuffers(cfg, N, dev) for _ in range(L)]
    counts_all = torch.zeros(L, E, dtype=torch.int32, device=dev)
    pop_all = torch.zeros(L, E, dtype=torch.int32, device=dev)
    for l, b in enumerate(bufs):
        b.counts = counts_all[l]
        b.pred_pop = pop_all[l]
    x_in = torch.zeros(L, N, H, dtype=torch.bfloat16, device=dev)
    host_counts = [torch.zeros(2, L, E, dtype=torch.int32).pin_memory() for _ in range(2)]

    def enqueue_token():
        # layer l's call gets, as a prefetch hint, what layer l-1's call predicted for it (section 4.3)
        for l in range(L):
            hint = bufs[l - 1].pred_ids if (l > 0 and N == 1 and args.hint) else None
            layer_forward(cfg, stack.layers[l], stack.layers[l + 1] if l + 1 < L else None, x_in[l], bufs[l],
                          hint_ids=hint)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        x_in.copy_(xs[0])
        enqueue_token()            # warm every kernel before capture
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            enqueue_token()
    torch.cuda.synchronize()

    # the cache: every expert resident (capacity = L*E), accounting only
    lib = B.lib()
    cache = lib.fate_cache_create(L, E, L * E, cfg.L_shallow, 0, 0, B.COPY_FN(0), None)
    stats = B.fate_cache_stats()
    tot = dict(hits=0, misses=0)
    evs = [torch.cuda.Event() for _ in range(2)]

    def account(slot):
        evs[slot].synchronize()
        hc = host_counts[slot]
        rc = lib.fate_expert_cache_step_layers(cache, 0, L, C.c_void_p(hc[0].data_ptr()),
                                               C.c_void_p(hc[1].data_ptr()), C.byref(stats))
        assert rc == 0, lib.fate_last_error()
        tot["hits"] += stats.n_hit_cache + stats.n_hit_prefetch
        tot["misses"] += stats.n_miss

    def run_tokens(n, first_step):
        for i in range(n):
            s = (first_step + i) % S
            x_in.copy_(xs[s], non_blocking=True)
            graph.replay()
            slot = i & 1
            host_counts[slot][0].copy_(counts_all, non_blocking=True)
            host_counts[slot][1].copy_(pop_all, non_blocking=True)
            evs[slot].record()
            if i > 0:
                account(slot ^ 1)
        if n > 0:
            account((n - 1) & 1)

    run_tokens(args.warmup, 0)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    run_tokens(args.steps, args.warmup)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / args.steps
    tok_s = args.steps * N / elapsed
    log(f"[bench] {args.steps} tokens in {elapsed * 1e3:.1f} ms -> {tok_s:.1f} tok/s")
    # a wait that ran out or an expert without weights inside the timed region voids the figure
    bad = [(l, b.status()) for l, b in enumerate(bufs) if b.status() != 0]
    if bad:
        raise SystemExit(f"bench.py: layer kernels reported a non-zero status word {bad}: the timing is not valid")

    # results of the graph path equal the eager chain (same inputs)
    x_in.copy_(xs[3]); graph.replay(); torch.cuda.synchronize()
    assert np.array_equal(bufs[5].ids.cpu().numpy(), t_ids[3, 5]), "graph replay diverged from the chain"

    # roofline of the dominant kernel pair (the layer kernel and its small reduction): they stream every
    # byte the layer needs (activated routed experts, the shared expert, both gate matrices, x, y)
    uniq = float(np.mean([len(set(t_ids[1, l].ravel().tolist())) for l in range(L)]))   # experts routed at the timed step
    layer_bytes = uniq * expert_bytes(H, cfg.I, cfg.bits, cfg.group) + \
        cfg.n_shared * expert_bytes(H, cfg.I_shared or 0, cfg.shared_bits, cfg.group) + 2 * E * H * 2 + N * H * (2 + 4)
    reps = 20
    blocker = torch.randn(8192, 8192, dtype=torch.float32, device=dev)   # keeps the queue busy while launches pile up
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    x_in.copy_(xs[1])
    for _ in range(3):
        torch.mm(blocker, blocker)
    e0.record()
    for _ in range(reps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    kern_us = e0.elapsed_time(e1) * 1e3 / (reps * L)
    achieved = layer_bytes / (kern_us * 1e-6) / 1e9
    log(f"[bench] layer kernel {kern_us:.2f} us/launch ({achieved:.0f} GB/s), layer algorithmic bytes "
        f"{layer_bytes / 1e6:.1f} MB")

    if args.calibrate_copy:
        # a plain device copy of known size, so that a counter run of this command can be scaled:
        # 5 copies of 1 GiB (reads 1 GiB, writes 1 GiB each)
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cpu = None
    if not args.no_cpu_baseline:
        ncores = len(os.sched_getaffinity(0))
        per, n_units, t_cpu = cpu_baseline_decode(cfg, xs, layers_sample=[0, 1, 6, 12, 18, 22],
                                                  tokens_sample=list(range(12 if qwen else 2)))
        cpu = {"value": 1.0 / (per * L), "unit": "tokens/s", "cores": min(ncores, blas_threads()),
               "kind": "oracle",
               "sample": f"{n_units} (token, layer) units of the same stack (layers 0, 1, 6, 12, 18, 22; decode steps 0-11), "
                         f"{t_cpu:.1f} s of oracle time, scaled to {L} layers per token"}
        log(f"[bench] oracle: {per:.2f} s per (token, layer) on the host")

    out = {
        "metric": "MoE-layer tokens/s (decode b=1, prefill 512) + % HBM / MFMA roofline",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int4 weights, bf16/fp16 activations, fp32 accumulate", "data": "synthetic",
        "config": {"workload": desc,
                   "step": f"one decode step of {N} token(s) through {L} MoE layers (route + predict + permute + FFN in "
                           "one launch per layer, cache step on the host)",
                   "layers": L, "batch": N, "decode_steps_cycled": S,
                   "layer_us": ms_per_step * 1e3 / L, "layer_algorithmic_MB": layer_bytes / 1e6,
                   "layer_hbm_frac": layer_bytes / (ms_per_step * 1e-3 / L) / 1e9 / HBM_PEAK_GBS,
                   "prediction_accuracy_topk": acc_k, "prediction_recall_topm": rec_m, "m": cfg.m,
                   "near_tie_rows": near_ties, "routed_rows": S * N * L,
                   "cache_hit_rate": tot["hits"] / max(1, tot["hits"] + tot["misses"])},
        "roofline": {"bound": "hbm",
                     "kernel": "moe_layer_decode_b1_kernel (one launch per layer)" if qwen else "moe_layer_decode_kernel + layer_reduce_kernel",
                     "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic("decode_qwen_b1_traffic.txt") if qwen else None,
                     "bytes_per_launch": layer_bytes, "us_per_launch": kern_us},
        "cpu_baseline": cpu,
    }
    if qwen and not args.no_prefill:
        # the metric's second figure: a 512-token prefill of the same model shape (its own weights: Zipf-skewed gate)
        del stack, graph, bufs
        torch.cuda.empty_cache()
        import copy
        pa = copy.copy(args)
        pa.workload, pa.steps, pa.warmup, pa.no_cpu_baseline, pa.layers = "qwen_prefill512", 10, 2, True, 0
        pre = bench_prefill(pa, emit=False)
        out["config"]["prefill512"] = {"tokens_per_s": pre["value"], "ms_per_pass": pre["ms_per_step"],
                                        "roofline": pre["roofline"], "ffn_mfma_frac": pre["config"]["ffn_mfma_frac"],
                                        "workload": pre["config"]["workload"]}
    print(json.dumps(out), flush=True)


DECODE_WORKLOADS = {
    # name: (shape, batch, decode steps cycled, description); every expert resident on the device
    "qwen_decode": ("qwen", 1, 128, "configs[1]: Qwen1.5-MoE-shaped decode, 24 layers chained, batch 1, "
                                    "60 experts top-4 (I=1408) + gated shared expert (I=5632), int4 g128"),
    "deepseek_decode8": ("deepseek", 8, 64, "configs[3]: DeepSeek-MoE-16B-shaped decode, 28 layers chained, batch 8, "
                                            "all experts resident"),
    "mixtral_decode": ("mixtral", 1, 128, "configs[4]: Mixtral-8x7B-shaped decode, 32 layers chained, batch 1, "
                                          "all experts resident"),
}

PREFILL_WORKLOADS = {
    # name: (shape, tokens, description)
    "qwen_prefill512": ("qwen_prefill", 512, "configs[2]: Qwen1.5-MoE-shaped prefill, 512 tokens, Zipf(1.1) routing"),
    "qwen_prefill2048": ("qwen_prefill", 2048, "configs[2]: Qwen1.5-MoE-shaped prefill, 2048 tokens, Zipf(1.1) routing"),
    "deepseek_prefill1024": ("deepseek", 1024, "configs[3]: DeepSeek-MoE-16B-shaped prefill, 1024 tokens, all experts resident"),
    "mixtral_prefill2048": ("mixtral", 2048, "configs[4]: Mixtral-8x7B-shaped prefill, 2048 tokens, all experts resident"),
}


def bench_prefill(args, emit=True):
    """One step = one prefill pass of N tokens through every layer of the stack
    (routing, prediction, permutation, MFMA expert FFN, cache accounting).
    emit=False: return the result instead of printing it (the decode run
    embeds the 512-token prefill figures of the metric)."""
    import numpy as np
    import torch
    import paper_2502_12224_amd.binding as B
    from paper_2502_12224_amd.stack import LayerBuffers, MoEStack, layer_forward
    from workloads import SHAPES

    shape, N, desc = PREFILL_WORKLOADS[args.workload]
    cfg = SHAPES[shape]
    dev = "cuda"
    L = args.layers or cfg.layers
    E, H = cfg.E, cfg.H
    t0 = time.time()
    log(f"[bench] {args.workload}: generating {L} layers on the device ...")
    stack = MoEStack(cfg, dev, layers=L, progress=lambda l: log(f"[bench]   layer {l} packed ({time.time() - t0:.0f}s)"))
    log(f"[bench] weights resident: {stack.nbytes() / 1e9:.2f} GB")
    xs, true_ids, pred_ids = stack.chain(N, 1)          # gate inputs of every layer (untimed chain)
    torch.cuda.synchronize()
    t_ids, p_ids = true_ids.cpu().numpy()[0], pred_ids.cpu().numpy()[0]
    from oracle import moe as O      # reporting (untimed): the oracle's definitions of the accuracy figures
    set_acc = float(np.mean([O.prefill_set_accuracy(p_ids[l], t_ids[l + 1]) for l in range(L - 1)])) if L > 1 else None
    tok_acc = float(np.mean([O.prediction_accuracy(p_ids[l], t_ids[l + 1], cfg.k)[0]
                             for l in range(L - 1)])) if L > 1 else None
    active = float(np.mean([len(set(t_ids[l].ravel())) for l in range(L)]))
    near_ties = 0
    for l in range(L):
        lw = stack.layers[l]
        z = O.gate_logits(xs[0, l].float().cpu().numpy(), lw.Wg.float().cpu().numpy(),
                          None if lw.bias is None else lw.bias.cpu().numpy())
        near_ties += len(O.near_tie_rows(z, cfg.k))

    bufs = [LayerBuffers(cfg, N, dev, mode=2) for _ in range(L)]
    counts_all = torch.zeros(L, E, dtype=torch.int32, device=dev)
    pop_all = torch.zeros(L, E, dtype=torch.int32, device=dev)
    for l, b in enumerate(bufs):
        b.counts = counts_all[l]
        b.pred_pop = pop_all[l]
    x_in = xs[0]

    def enqueue_pass():
        for l in range(L):
            layer_forward(cfg, stack.layers[l], stack.layers[l + 1] if l + 1 < L else None, x_in[l], bufs[l])

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        enqueue_pass()
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            enqueue_pass()
    torch.cuda.synchronize()
    lib = B.lib()
    cache = lib.fate_cache_create(L, E, L * E, cfg.L_shallow, 0, 0, B.COPY_FN(0), None)
    stats = B.fate_cache_stats()
    host_counts = torch.zeros(2, L, E, dtype=torch.int32).pin_memory()
    hits = misses = 0

    def one_pass():
        nonlocal hits, misses
        graph.replay()
        host_counts[0].copy_(counts_all, non_blocking=True)
        host_counts[1].copy_(pop_all, non_blocking=True)
        torch.cuda.current_stream().synchronize()
        rc = lib.fate_expert_cache_step_layers(cache, 0, L, C.c_void_p(host_counts[0].data_ptr()),
                                               C.c_void_p(host_counts[1].data_ptr()), C.byref(stats))
        assert rc == 0, lib.fate_last_error()
        hits += stats.n_hit_cache + stats.n_hit_prefetch
        misses += stats.n_miss

    for _ in range(args.warmup):
        one_pass()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        one_pass()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / args.steps
    tok_s = args.steps * N / elapsed
    log(f"[bench] {args.steps} passes of {N} tokens x {L} layers in {elapsed * 1e3:.1f} ms -> {tok_s:.0f} tok/s")
    bad = [(l, int(b.ffn_ws[:4].view(torch.int32)[0])) for l, b in enumerate(bufs)
           if int(b.ffn_ws[:4].view(torch.int32)[0]) != 0]
    if bad:
        raise SystemExit(f"bench.py: the FFN reported a non-zero status word {bad}: the timing is not valid")

    if args.calibrate_copy:
        # a plain device copy of known size, so that a counter run of this command can be scaled
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # roofline of the dominant kernel: the up/gate grouped GEMM (2/3 of the FLOPs)
    up_flops = 4.0 * H * (N * cfg.k * cfg.I + N * cfg.n_shared * (cfg.I_shared or 0))
    layer_flops = 1.5 * up_flops
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    times = []
    for phase in (1, 0):
        reps = 3
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            for l in range(L):
                a = (x_in[l], stack.layers[l].table, bufs[l].counts, bufs[l].offsets, bufs[l].perm, bufs[l].inv_perm,
                     bufs[l].order, bufs[l].w, stack.layers[l].shared_table, stack.layers[l].shared_gate, bufs[l].y,
                     bufs[l].ffn_ws)
                if phase:
                    B.fate_profile_ffn_mfma_phase(bufs[l].desc, phase, *a)
                else:
                    B.fate_moe_ffn_q(bufs[l].desc, *a)
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) * 1e3 / (reps * L))
    up_us, ffn_us = times
    achieved = up_flops / (up_us * 1e-6) / 1e12
    # the other roof: the stored bytes of the experts the layer activates (codes + scales), once per layer
    layer_bytes = active * expert_bytes(H, cfg.I, cfg.bits, cfg.group) + \
        cfg.n_shared * expert_bytes(H, cfg.I_shared or 0, cfg.shared_bits, cfg.group)
    hbm_gbs = layer_bytes / (ffn_us * 1e-6) / 1e9
    log(f"[bench] prep+up GEMM {up_us:.1f} us/layer ({achieved:.0f} TFLOP/s), whole FFN {ffn_us:.1f} us/layer "
        f"({layer_flops / (ffn_us * 1e-6) / 1e12:.0f} TFLOP/s; {layer_bytes / 1e6:.1f} MB of weights -> {hbm_gbs:.0f} GB/s)")

    cpu = None
    if not args.no_cpu_baseline and L > 1:
        rows = list(range(0, N, max(1, N // 128)))[:128]
        t_route, t_ffn = cpu_baseline_prefill(cfg, x_in[0], 0, rows)
        per_token = t_route / N + t_ffn / len(rows)
        cpu = {"value": 1.0 / (per_token * L), "unit": "tokens/s",
               "cores": min(len(os.sched_getaffinity(0)), blas_threads()), "kind": "oracle",
               "sample": f"layer 0: routing, prediction and permutation of all {N} tokens ({t_route:.2f} s) and the "
                         f"FFN of {len(rows)} token rows ({t_ffn:.1f} s, includes dequantising their experts), "
                         f"scaled per token to {L} layers"}
        log(f"[bench] oracle: {per_token:.3f} s per (token, layer) on the host")

    out = {
        "metric": "MoE-layer tokens/s (decode b=1, prefill 512) + % HBM / MFMA roofline",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int4/int8 weights dequantised to fp16, fp16 MFMA, fp32 accumulate", "data": "synthetic",
        "config": {"workload": desc, "step": f"one prefill pass of {N} tokens through {L} MoE layers",
                   "layers": L, "tokens": N, "layer_us": ms_per_step * 1e3 / L,
                   "layer_useful_GFLOP": layer_flops / 1e9, "ffn_call_us": ffn_us,
                   "ffn_mfma_frac": layer_flops / (ffn_us * 1e-6) / 1e12 / MFMA_PEAK_TFLOPS,
                   "experts_active_per_layer": active, "prefill_set_accuracy": set_acc,
                   "prediction_accuracy_topk_per_token": tok_acc, "near_tie_rows": near_ties, "routed_rows": N * L,
                   "cache_hit_rate": hits / max(1, hits + misses)},
        "roofline": {"bound": "mfma", "kernel": "prefill_prep_kernel + grouped_gemm_kernel<2>", "achieved": achieved,
                     "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_PEAK_TFLOPS,
                     "traffic": measured_traffic(f"prefill_{args.workload}_traffic.txt"),
                     "flops_per_launch": up_flops, "us_per_launch": up_us,
                     "hbm_roof": {"bound": "hbm", "kernel": "whole FFN call (four launches)",
                                  "achieved": hbm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                  "frac": hbm_gbs / HBM_PEAK_GBS, "bytes_per_layer": layer_bytes,
                                  "us_per_layer": ffn_us}},
        "cpu_baseline": cpu,
    }
    if not emit:
        return out
    print(json.dumps(out), flush=True)


OFFLOAD_WORKLOADS = {
    # name: (shape, prefill tokens, decode batch, decode steps, description)
    "deepseek_offload": ("deepseek", 1024, 8, 64,
                         "configs[3]: DeepSeek-MoE-16B-shaped, routed experts in pinned host memory, 30% of them "
                         "cached on the device (3 shallow layers full); prefill 1024 tokens, then decode batch 8"),
    "mixtral_offload": ("mixtral", 2048, 1, 128,
                        "configs[4]: Mixtral-8x7B-shaped, experts in pinned host memory, 25% cached on the device; "
                        "prefill 2048 tokens, then decode batch 1"),
}


def h2d_peak_gbs(dev):
    """Pinned host -> device copy rate of this machine (256 MiB, best of 5)."""
    import torch
    src = torch.empty(256 << 20, dtype=torch.uint8, pin_memory=True)
    dst = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best = 0.0
    for _ in range(5):
        e0.record(); dst.copy_(src, non_blocking=True); e1.record(); torch.cuda.synchronize()
        best = max(best, src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    return best


def bench_offload(args):
    """Offloaded stack: one step = one decode step of the batch through every
    layer (route, predict, permute, cache step with H2D copies on the side
    stream, FFN).  The prefill pass that fills the cache is timed separately and
    reported in config."""
    import torch
    import paper_2502_12224_amd.binding as B
    from paper_2502_12224_amd.stack import LayerBuffers, OffloadedStack
    from workloads import SHAPES, chain_next_hidden, gen_hidden, unit_rmsnorm_bf16

    import dataclasses
    shape, Np, Nd, S, desc = OFFLOAD_WORKLOADS[args.workload]
    cfg = SHAPES[shape]
    if args.routed_bits:
        cfg = dataclasses.replace(cfg, bits=args.routed_bits)       # ablation: experts moved and cached at 8 bits
    dev = "cuda"
    L = args.layers or cfg.layers
    E, H = cfg.E, cfg.H
    steps = args.steps
    mode = args.mode
    cache_frac = cfg.cache_frac if args.cache_frac is None else args.cache_frac
    cache_total = 0 if mode == "lod" else int(cache_frac * L * E)
    lib = B.lib()
    ebytes = expert_bytes(H, cfg.I, cfg.bits, cfg.group)
    peak = h2d_peak_gbs(dev)
    t_expert = ebytes / (peak * 1e9)
    t0 = time.time()
    log(f"[bench] {args.workload}: {L} layers x {E} experts of {ebytes / 1e6:.2f} MB -> pinned host pool "
        f"{L * E * ebytes / 1e9:.1f} GB; cache_total {cache_total}, H2D peak {peak:.1f} GB/s")
    st = OffloadedStack(cfg, cache_total, 0, staging_slots=3 * E, device=dev, layers=L,
                        predictor={"fate": "gate", "eap": "eap", "lod": "none"}[mode],
                        low_bits=2 if args.low_percent > 0 else 0,
                        progress=lambda l: log(f"[bench]   layer {l} in the host pool ({time.time() - t0:.0f}s)"))
    log(f"[bench] per-layer capacities {st.caps}")

    def run(N, nsteps, first_step, buf):
        for s in range(nsteps):
            h = gen_hidden(cfg, N, step=first_step + s, device=dev).to(torch.float32)
            for l in range(L):
                x = unit_rmsnorm_bf16(h)
                y = st.layer(l, x, buf)
                h = chain_next_hidden(h, y)

    def snapshot():
        d = dict(st.stats)
        d["bytes"] = st.bytes_copied()
        return d

    def phase(N, nsteps, first_step, buf):
        torch.cuda.synchronize()
        a = snapshot()
        t = time.perf_counter()
        run(N, nsteps, first_step, buf)
        torch.cuda.synchronize()
        el = time.perf_counter() - t
        b = snapshot()
        d = {k: b[k] - a[k] for k in a}
        hits = d["hit_cache"] + d["hit_prefetch"]
        return dict(seconds=el, tokens_per_s=N * nsteps / el, hit_rate=hits / max(1, hits + d["miss"]),
                    hit_rate_cache_only=d["hit_cache"] / max(1, hits + d["miss"]),
                    pair_hit_rate=d["pair_hits"] / max(1, d["pair_hits"] + d["pair_misses"]),
                    h2d_GB=d["bytes"] / 1e9, h2d_GBs=d["bytes"] / el / 1e9, prefetch_issued=d["prefetch"],
                    prefetch_wasted=d["wasted"], demand_loads=d["miss"])

    pbuf = LayerBuffers(cfg, Np, dev)
    dbuf = LayerBuffers(cfg, Nd, dev)
    run(Nd, 1, 10_000, dbuf)                 # warm the kernels and the copy path
    # Calibration of the decode prefetch cap (section 4.3): T is the compute time of a layer whose experts
    # are all on the device - layer 0 is fully cached, so its calls issue no copy - and n = floor(T / t_expert).
    t_layer_resident, n_cal = None, None
    if st.caps[0] == E:
        xcal = unit_rmsnorm_bf16(gen_hidden(cfg, Nd, step=30_000, device=dev).to(torch.float32))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            st.layer(0, xcal, dbuf)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(20):
            st.layer(0, xcal, dbuf)
        e1.record()
        torch.cuda.synchronize()
        t_layer_resident = e0.elapsed_time(e1) * 1e-3 / 20
        n_cal = lib.fate_n_max_from_times(t_layer_resident, 0.0, 0.0, t_expert)
        log(f"[bench] resident layer {t_layer_resident * 1e6:.1f} us, one expert over the link "
            f"{t_expert * 1e6:.1f} us -> n = {n_cal}")
    n_max = 0 if mode == "lod" else (args.n_max if args.n_max is not None else (n_cal or 0))
    log(f"[bench] mode {mode}, decode prefetch cap {n_max}")
    if mode == "eap":
        # the baseline's statistics: co-activation counts over calibration decode steps (untimed, no prefetch)
        st.eap_learning = True
        run(Nd, args.eap_calibration_steps, 40_000, dbuf)
        st.eap_learning = False
    B._check(lib.fate_cache_set_n_max(st.cache, 0 if mode == "lod" else E))   # prefill: every predicted expert, most popular first
    st.overlap_piece = args.overlap_piece        # prefill FFN in pieces that follow the transfers (0 = one call per layer)
    if args.low_percent > 0:
        st.set_low_percent(args.low_percent)     # prefill only: the least popular predicted experts move as 2-bit copies
    pre = phase(Np, 1, 20_000, pbuf)
    if args.low_percent > 0:
        st.set_low_percent(0)
    B._check(lib.fate_cache_set_n_max(st.cache, n_max))
    log(f"[bench] prefill {Np} tokens: {pre['seconds'] * 1e3:.1f} ms, {pre['tokens_per_s']:.0f} tok/s, "
        f"hit rate {pre['hit_rate']:.3f}, H2D {pre['h2d_GB']:.2f} GB at {pre['h2d_GBs']:.1f} GB/s")
    run(Nd, args.warmup, 0, dbuf)
    dec = phase(Nd, steps, args.warmup, dbuf)
    log(f"[bench] decode batch {Nd} x {steps} steps: {dec['tokens_per_s']:.1f} tok/s, hit rate {dec['hit_rate']:.3f} "
        f"(cache only {dec['hit_rate_cache_only']:.3f}), H2D {dec['h2d_GB']:.2f} GB at {dec['h2d_GBs']:.1f} GB/s")
    out = {
        "metric": "MoE-layer tokens/s (decode b=1, prefill 512) + % HBM / MFMA roofline",
        "value": dec["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": dec["seconds"] * 1e3 / steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int4/int8 weights, bf16/fp16 activations, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": desc, "step": f"one decode step of batch {Nd} through {L} MoE layers, experts offloaded",
                   "layers": L, "batch": Nd, "mode": mode, "routed_bits": cfg.bits, "cache_frac": cache_frac,
                   "prefill_low_width_percent": args.low_percent, "prefill_overlap_piece": args.overlap_piece,
                   "cache_total": cache_total, "layer_capacities": st.caps,
                   "n_max": n_max, "n_from_resident_layer_time": n_cal,
                   "t_layer_resident_us": None if t_layer_resident is None else t_layer_resident * 1e6,
                   "t_expert_us": t_expert * 1e6,
                   "decode": dec, "prefill": dict(tokens=Np, **pre)},
        "roofline": {"bound": "pcie", "kernel": "side-stream H2D copies of missed / prefetched experts",
                     "achieved": dec["h2d_GBs"], "peak": peak, "unit": "GB/s", "frac": dec["h2d_GBs"] / peak,
                     "traffic": None, "peak_source": "256 MiB pinned copy measured in this run"},
        "cpu_baseline": None,
    }
    st.close()
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=0, help="prefill workloads: use only the first LAYERS layers")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="default 256 (decode) / 10 (prefill)")
    ap.add_argument("--warmup", type=int, default=None, help="default 32 (decode) / 2 (prefill)")
    ap.add_argument("--workload", default="qwen_decode")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefill", action="store_true",
                    help="decode: skip the 512-token prefill figures that the default run adds to its line")
    ap.add_argument("--hint", action="store_true",
                    help="decode: hand layer l the previous layer's prediction as a prefetch hint (measured slower "
                         "at this prediction accuracy: a wrong hint costs a second pass)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="decode: also run five 1 GiB device copies (reference for hardware-counter runs)")
    ap.add_argument("--mode", default="fate", choices=["fate", "eap", "lod"],
                    help="offload workloads: fate = cross-layer gate prediction + shallow-favoring cache (the method); "
                         "eap = same cache, activation-path prediction; lod = no cache, no prefetch (load on demand)")
    ap.add_argument("--cache-frac", type=float, default=None,
                    help="offload workloads: fraction of the routed experts cached on the device (default: the configuration's)")
    ap.add_argument("--routed-bits", type=int, default=0, choices=[0, 4, 8],
                    help="offload workloads: code width of the routed experts (ablation of the quantisation step)")
    ap.add_argument("--eap-calibration-steps", type=int, default=32)
    ap.add_argument("--overlap-piece", type=int, default=0,
                    help="offload workloads: prefill FFN in pieces of this many experts that follow the order of the "
                         "transfers (experts in the cache first), each piece waiting only for its own copies; 0 = one call")
    ap.add_argument("--low-percent", type=int, default=0,
                    help="offload workloads: share of the predicted experts, least popular first, that the prefill pass "
                         "moves as 2-bit copies (popularity-aware hybrid width; the paper uses 25 for Qwen1.5-MoE)")
    ap.add_argument("--n-max", type=int, default=None,
                    help="offload workloads: cap on prefetched experts per layer in decode (default: n = floor(T / "
                         "t_expert) from the measured resident layer time and link rate)")
    args = ap.parse_args()
    decode = args.workload in DECODE_WORKLOADS
    if args.steps is None:
        args.steps = 256 if decode else OFFLOAD_WORKLOADS[args.workload][3] if args.workload in OFFLOAD_WORKLOADS else 10
    if args.warmup is None:
        args.warmup = 32 if decode else 2
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); the multi-GPU sharding is design-only.",
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback.", file=sys.stderr)
        sys.exit(3)
    if args.workload in DECODE_WORKLOADS:
        bench_decode(args)
    elif args.workload in PREFILL_WORKLOADS:
        bench_prefill(args)
    elif args.workload in OFFLOAD_WORKLOADS:
        bench_offload(args)
    else:
        print(f"bench.py: unknown workload {args.workload}; choose one of "
              f"{sorted(DECODE_WORKLOADS) + sorted(PREFILL_WORKLOADS) + sorted(OFFLOAD_WORKLOADS)}", file=sys.stderr)
        sys.exit(2)


if __name__ == "__main__":
    main()
