#!/usr/bin/env python3
"""Benchmark of the slim-attention decode step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N] [--variant auto]

A step is one pass of the whole hot path (`slim_decode`: scores, softmax, weighted sum of K,
split merge, per-head W_KV projection) over one batch of the seeded synthetic workload, with
every input resident in HBM before the timed region.  The default workload is config 2, the
largest one that fits one GPU (Phi-3-mini-shaped batch, B=16, H=32, d=3072, ragged contexts of
8192..32768 rows, bf16 K-cache); config 1 (CodeLlama-7B-shaped, B=1, T=16384) is timed in the same
run and nested in the same line.  The K-cache and W_KV are rotated over several identical copies so
the 256 MB memory-side cache cannot serve them.

Prints one JSON line: whole-job tokens/s (a token = one sequence's decode step through this
one attention layer), the same-GPU `vanilla_kv_decode` time, the roofline entry of the
dominant kernel (algorithmic bytes / measured kernel time, HIP events on the launch stream),
and the CPU oracle timed on the host cores as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
STAGES = {                      # kernels of one slim_decode call, in launch order, per variant
    "generic": ["head_scores", "weighted_sum", "combine", "project"],
    "fused": ["fused_stream", "project_mfma"],          # one launch when B <= 16: the second entry stays 0
    "fused_split": ["fused_stream", "project_mfma"],
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(config_index, kernel):
    """HBM bytes per launch of `kernel` on this workload, as measured with rocprofv3 --pmc
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size); recorded in the counter summary
    under profiles/.  None when no measurement of this workload is on record."""
    import glob
    import re
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*pmc*.txt"))):
        m = re.search(rf"^traffic_bytes_per_launch configs\[{config_index}\] {re.escape(kernel)} = (\d+)", open(path).read(), re.M)
        if m:
            return int(m.group(1))
    return None


def timed(torch, fn, steps, warmup):
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    t = time.perf_counter()
    for i in range(steps):
        fn(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t) * 1e3 / steps


def calibration_copy(args, torch):
    """--calibration-copy: five plain 128 MiB device copies, a kernel of known traffic for scaling byte counters."""
    if not args.calibration_copy:
        return
    src = torch.empty(128 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


XCACHE_STAGES = ["q_tilde (head_scores on W_K)", "dense_scores", "weighted_sum", "combine", "project"]
XCACHE_MFMA_STAGES = ["xq_tilde", "xscores", "xweighted", "project_mfma"]     # two passes over X
XCACHE_ONEPASS_STAGES = ["xq_tilde", "xfused", "project_mfma"]               # 512 <= d_model <= 1280


def bench_xcache(args, cfg, torch, binding, synth, emit=True):
    """configs[4]: the X-cache scheme for projection width e > d_model (absorbed form)."""
    B, H, T, dm, d_k, e = cfg.B, cfg.H, cfg.T, cfg.d, cfg.d_k, cfg.e
    log(f"[bench] building inputs for config {cfg.index} ({cfg.name}) ...")
    p = synth.make_problem(cfg)
    Xh = np.stack([synth.to_storage(sq.X, cfg.dtype) for sq in p.seqs])
    to_device = binding.to_device
    ncopies = args.copies or max(2, int(np.ceil(512e6 / Xh.nbytes)) + 1)
    Xs = [to_device(Xh) for _ in range(ncopies)]
    q = to_device(p.q.astype(np.float32))
    Wk = to_device(binding.slim_pack_weights(p.w.W_K, cfg.dtype))
    Wv = to_device(binding.slim_pack_weights(p.w.W_V, cfg.dtype))
    out = torch.zeros((B, e), device="cuda", dtype=torch.float32)

    # --variant fused_split: scores and weighted sum as two passes over X; generic: the plain kernels
    variant = {"auto": binding.VARIANT_AUTO, "generic": binding.VARIANT_GENERIC,
               "fused": binding.VARIANT_FUSED, "fused_split": binding.VARIANT_FUSED_SPLIT}[args.variant]

    def slim(i, **extra):
        binding.slim_decode_xcache(q, Xs[i % ncopies], Wk, Wv, out, B, H, T, dm, d_k, dtype=cfg.dtype, variant=variant, **extra)

    calibration_copy(args, torch)
    log("[bench] timing slim_decode_xcache ...")
    ms = timed(torch, slim, args.steps, args.warmup)
    # the same-GPU comparison reads e-wide K and V caches (random values: only the traffic matters)
    Kr = torch.randn((B, T, e), device="cuda").to(torch.bfloat16)
    Vr = torch.randn((B, T, e), device="cuda").to(torch.bfloat16)
    out_v = torch.zeros_like(out)
    log("[bench] timing vanilla_kv_decode on e-wide K and V ...")
    ms_van = timed(torch, lambda i: binding.vanilla_kv_decode(q, Kr, Vr, out_v, B, H, T, e, dtype=cfg.dtype),
                   max(5, args.steps // 10), 3)
    del Kr, Vr
    stage = binding.new_stage_buffer()
    acc = np.zeros(binding.MAX_STAGES)
    for i in range(args.steps):
        slim(i, stage_ms=stage)
        acc += np.array(list(stage))
    acc /= args.steps
    # three launches: q~, the one-pass kernel, projection; four: two passes over X; five: the plain kernels
    names = XCACHE_ONEPASS_STAGES if acc[3] == 0.0 else (XCACHE_MFMA_STAGES if acc[4] == 0.0 else XCACHE_STAGES)
    dom = int(np.argmax(acc[:len(names)]))
    # dense contractions over all heads: priced against the bf16 MFMA peak with the method's own
    # flop counts (the hi + lo split of q~ doubles the MFMA work of the scores; not counted)
    dense = 2.0 * B * H * T * dm
    flops = {"xscores": dense, "xweighted": dense, "dense_scores": dense, "weighted_sum": dense,
             "xfused": 2.0 * dense}.get(names[dom], 2.0 * B * dm * e)
    achieved = flops / (acc[dom] * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": names[dom], "achieved": round(achieved, 2), "peak": 2500.0, "unit": "TFLOP/s",
                "frac": round(achieved / 2500.0, 5), "traffic": measured_traffic(cfg.index, names[dom]), "kernel_ms": round(float(acc[dom]), 5),
                "algorithmic_flops": flops,
                "stage_ms": {n: round(float(acc[i]), 5) for i, n in enumerate(names)}}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import mha_oracle as orc
        log("[bench] timing the CPU oracle on sequence 0 (builds the e-wide K and V, then the decode step) ...")
        t0, c0 = time.perf_counter(), os.times()
        ref0 = orc.vanilla_decode_from_x(p.q[0], p.seqs[0].X, p.w.W_K, p.w.W_V, H)
        wall = time.perf_counter() - t0
        c1 = os.times()
        busy = (c1.user - c0.user) + (c1.system - c0.system)
        slim(0)
        torch.cuda.synchronize()
        got0 = out[0].cpu().numpy().astype(np.float64).reshape(H, d_k)
        r0 = ref0.reshape(H, d_k)
        err = float((np.abs(got0 - r0).max(axis=1) / np.abs(r0).max(axis=1)).max())
        cpu = {"value": round(1.0 / wall, 4), "unit": "tokens/s", "cores": max(1, int(round(busy / wall))), "kind": "oracle",
               "host_cores": os.cpu_count(),
               "sample": f"sequence 0 of config {cfg.index} ({T} rows x {dm}), one fp64 evaluation including K = X W_K, V = X W_V (e = {e})",
               "gpu_max_rel_err_vs_oracle_seq0": float(f"{err:.3e}")}
    x_bytes = float(B) * T * dm * 2
    result = {
        "metric": "decode tokens/s (one attention layer step, X-cache: K and V never stored), 1 GPU",
        "value": round(B / (ms * 1e-3), 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{cfg.index}] {cfg.name}", "B": B, "H": H, "d_model": dm, "d_k": d_k, "e": e, "T": T,
                   "x_cache_copies_rotated": ncopies},
        "x_cache_gbps": round(x_bytes / (ms * 1e-3) / 1e9, 1),
        "algorithmic_bytes_gbps": round((x_bytes + 2.0 * dm * e * 2) / (ms * 1e-3) / 1e9, 1),
        "vanilla_kv_ms_per_step": round(ms_van, 5), "speedup_vs_vanilla_kv": round(ms_van / ms, 3),
        "roofline": roofline, "cpu_baseline": cpu,
    }
    if emit:
        print(json.dumps(result), flush=True)
    return result


def bench_ecache_layers(args, cfg, torch, binding, synth):
    """--ecache --layers L (config 3): L decoder layers' cross-attention in a row, three ways.  Option 2 of the
    encoder-decoder section: every layer reads the SAME encoder output E through slim_decode_xcache with its
    own W_K, W_V.  Option 1: every layer reads its own K-cache through slim_decode with its own W_KV.  Vanilla:
    its own K and V caches.  Values are random (only shapes and traffic matter here; parity is the tests' job)."""
    B, H, T, d, d_k = cfg.B, cfg.H, cfg.T, cfg.d, cfg.d_k
    L = args.layers
    gen = torch.Generator(device="cuda").manual_seed(20250305)
    rnd = lambda *shape, std=1.0: (torch.randn(shape, device="cuda", generator=gen) * std).to(torch.bfloat16)
    E = rnd(B, T, d)
    Wk = [rnd(d, d, std=d ** -0.5) for _ in range(L)]
    Wv = [rnd(d, d, std=d ** -0.5) for _ in range(L)]
    Wkv = [rnd(d, d) for _ in range(L)]
    Ks = [rnd(B, T, d, std=(1.75 / d) ** 0.5) for _ in range(L)]
    Vs = [rnd(B, T, d, std=d ** -0.5) for _ in range(L)]
    q = torch.randn((B, d), device="cuda", generator=gen)
    out = torch.zeros((B, d), device="cuda", dtype=torch.float32)
    ws = torch.empty(max(binding.slim_workspace_bytes(B, H, T, d, "bf16"), binding.slim_workspace_bytes_xcache(B, H, T, d, d_k, "bf16")),
                     dtype=torch.uint8, device="cuda")
    binding.slim_init()

    def option2(i):
        for l in range(L):
            binding.slim_decode_xcache(q, E, Wk[l], Wv[l], out, B, H, T, d, d_k, dtype="bf16", workspace=ws)

    def option1(i):
        for l in range(L):
            binding.slim_decode(q, Ks[l], Wkv[l], out, B, H, T, d, dtype="bf16", workspace=ws)

    def vanilla(i):
        for l in range(L):
            binding.vanilla_kv_decode(q, Ks[l], Vs[l], out, B, H, T, d, dtype="bf16", workspace=ws)

    steps, warm = max(3, args.steps // 10), 2
    ms2 = timed(torch, option2, steps, warm) / L
    ms1 = timed(torch, option1, steps, warm) / L
    msv = timed(torch, vanilla, steps, warm) / L
    e_bytes = float(B) * T * d * 2
    result = {
        "metric": "per-layer time of the cross-attention decode step over L decoder layers: E-cache (option 2) vs K-only cache (option 1) vs K+V, 1 GPU",
        "value": round(B / (ms2 * 1e-3), 2), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warm,
        "ms_per_step": round(ms2, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"configs[3] {cfg.name}, {L} layers on one shared E", "B": B, "H": H, "d": d, "d_k": d_k, "T": T, "layers": L},
        "ecache_option2_ms_per_layer": round(ms2, 5), "kcache_option1_ms_per_layer": round(ms1, 5),
        "vanilla_kv_ms_per_layer": round(msv, 5),
        "cache_bytes_per_layer": {"option2_E_shared": e_bytes / L, "option1_K": e_bytes, "vanilla_KV": 2 * e_bytes},
        "roofline": {"bound": "hbm", "kernel": "all launches of one layer (option 2)", "achieved": round((e_bytes + 2.0 * d * d * 2) / (ms2 * 1e-3) / 1e9, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round((e_bytes + 2.0 * d * d * 2) / (ms2 * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                     "traffic": None},
        "cpu_baseline": None,
    }
    print(json.dumps(result), flush=True)


def bench_block(args, cfg, torch, binding, synth):
    """--block: one generated token per sequence through the whole attention block
    (slim_attention_block: q and k projections, append, decode step, W_O) against
    vanilla_attention_block (q, k, v projections, append to both caches, K+V decode, W_O)."""
    B, H, T, d, d_k = cfg.B, cfg.H, cfg.T, cfg.d, cfg.d_k
    es = 2 if cfg.dtype == "bf16" else 4
    log(f"[bench] building inputs for the attention block on config {cfg.index} ({cfg.name}) ...")
    p = synth.make_problem(cfg)
    lens = p.lengths                                   # rows after the append
    W_O = synth.make_w_o(cfg)
    el = np.uint16 if cfg.dtype == "bf16" else np.float32
    Kh = np.zeros((B, T, d), dtype=el)
    Vh = np.zeros((B, T, d), dtype=el)
    K64 = V64 = None
    for b, sq in enumerate(p.seqs):
        n = int(lens[b]) - 1
        Kb = synth.project_cache(sq.X[:n], p.w.W_K)
        Vb = synth.project_cache(sq.X[:n], p.w.W_V)
        Kh[b, :n] = synth.to_storage(Kb, cfg.dtype)
        Vh[b, :n] = synth.to_storage(Vb, cfg.dtype)
        if b == 0:
            K64, V64 = Kb, Vb
        sq.X = None
    wkv, _ = binding.slim_prepare_wkv(p.w.W_K, p.w.W_V)
    to_device = binding.to_device
    pack = lambda W: to_device(binding.slim_pack_weights(W, cfg.dtype))
    ncopies = args.copies or max(2, int(np.ceil(512e6 / Kh.nbytes)) + 1)
    Ks = [to_device(Kh) for _ in range(ncopies)]
    Vs = [to_device(Vh) for _ in range(ncopies)]
    # the weights rotate too: at small batch they are as many bytes as the cache
    wcopies = max(2, int(np.ceil(512e6 / (4.0 * d * d * es))) + 1)
    Wq, Wk, Wv, Wo, Wkv = ([pack(W) for _ in range(wcopies)] for W in (p.w.W_Q, p.w.W_K, p.w.W_V, W_O, wkv))
    x = to_device(np.stack([sq.x for sq in p.seqs]).astype(np.float32))
    y = torch.zeros((B, d), device="cuda", dtype=torch.float32)
    y_v = torch.zeros_like(y)
    ws = torch.empty(binding.slim_workspace_bytes_block(B, H, T, d, cfg.dtype), dtype=torch.uint8, device="cuda")
    kw = dict(dtype=cfg.dtype, workspace=ws)
    if bool((lens != T).any()):
        kw.update(seq_lens=torch.from_numpy(lens).cuda(), seq_lens_host=lens)
    if args.rope:
        kw["rope_table"] = to_device(binding.slim_rope_table(T, d_k, 10000.0))

    def slim(i, **extra):
        j = i % wcopies
        binding.slim_attention_block(x, Wq[j], Wk[j], Wkv[j], Wo[j], Ks[i % ncopies], y, B, H, T, d, **kw, **extra)

    def vanilla(i, **extra):
        j = i % wcopies
        binding.vanilla_attention_block(x, Wq[j], Wk[j], Wv[j], Wo[j], Ks[i % ncopies], Vs[i % ncopies], y_v,
                                        B, H, T, d, **kw, **extra)

    log("[bench] timing slim_attention_block ...")
    ms_slim = timed(torch, slim, args.steps, args.warmup)
    log("[bench] timing vanilla_attention_block ...")
    ms_van = timed(torch, vanilla, args.steps, args.warmup)
    stage = binding.new_stage_buffer()
    acc, vacc = np.zeros(3), np.zeros(3)
    for i in range(args.steps):
        slim(i, stage_ms=stage)
        acc += np.array(list(stage))[:3]
        vanilla(i, stage_ms=stage)
        vacc += np.array(list(stage))[:3]
    acc /= args.steps
    vacc /= args.steps
    names = ["projections_in + append", "decode step", "projection_out"]
    k_bytes = float(lens.astype(np.int64).sum()) * d * es
    w_bytes = float(d) * d * es
    alg_bytes = k_bytes + 4 * w_bytes                  # K once, W_Q, W_K, W_KV, W_O once
    achieved = alg_bytes / (ms_slim * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "whole block (all launches of one slim_attention_block call)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None, "algorithmic_bytes": alg_bytes,
                "kernel_ms": round(ms_slim, 5),
                "stage_ms": {n: round(float(acc[i]), 5) for i, n in enumerate(names)},
                "vanilla_stage_ms": {n: round(float(vacc[i]), 5) for i, n in enumerate(names)}}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import mha_oracle as orc
        log("[bench] timing the CPU oracle (attention_block on sequence 0, fp64 K and V resident) ...")
        x0 = p.seqs[0].x
        base = 10000.0 if args.rope else None
        ref0, _, _ = orc.attention_block(x0, K64, V64, p.w.W_Q, p.w.W_K, p.w.W_V, W_O, H, base)
        slim(0)
        torch.cuda.synchronize()
        got0 = y[0].cpu().numpy().astype(np.float64)
        err = float(np.abs(got0 - ref0).max() / np.abs(ref0).max())
        reps, t0c, c0 = 0, time.perf_counter(), os.times()
        while reps < 3 or (time.perf_counter() - t0c < 10.0 and reps < 200):
            orc.attention_block(x0, K64, V64, p.w.W_Q, p.w.W_K, p.w.W_V, W_O, H, base)
            reps += 1
        wall = time.perf_counter() - t0c
        c1 = os.times()
        busy = (c1.user - c0.user) + (c1.system - c0.system)
        cpu = {"value": round(reps / wall, 3), "unit": "tokens/s", "cores": max(1, int(round(busy / wall))),
               "kind": "oracle", "host_cores": os.cpu_count(),
               "sample": f"sequence 0 of config {cfg.index} ({int(lens[0]) - 1} cached rows x {d}), {reps} repeats of the fp64 attention block",
               "gpu_max_rel_err_vs_oracle_seq0": float(f"{err:.3e}")}
    result = {
        "metric": "decode tokens/s (one whole attention block per token: projections, append, K-cache-only decode step, W_O) vs the vanilla K+V block, 1 GPU",
        "value": round(B / (ms_slim * 1e-3), 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_slim, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{cfg.index}] {cfg.name} + whole attention block" + (" + rotary keys" if args.rope else ""),
                   "B": B, "H": H, "d": d, "d_k": d_k, "T": T, "sum_len": int(lens.sum()),
                   "k_cache_copies_rotated": ncopies, "weight_copies_rotated": wcopies},
        "vanilla_block_ms_per_step": round(ms_van, 5), "speedup_vs_vanilla_block": round(ms_van / ms_slim, 3),
        "bytes_ratio_vanilla_over_slim": round((2 * k_bytes + 4 * w_bytes) / alg_bytes, 3),
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(result), flush=True)


def bench_kcache(args, cfg, torch, binding, synth, with_cpu):
    """One K-cache config: slim_decode against vanilla_kv_decode, per-kernel times, the read probe and
    (with_cpu) the oracle on the host cores.  Returns the result as a dict."""
    B, H, T, d, d_k = cfg.B, cfg.H, cfg.T, cfg.d, cfg.d_k
    es = 2 if cfg.dtype == "bf16" else 4
    log(f"[bench] building inputs for config {cfg.index} ({cfg.name}) ...")
    t0 = time.time()
    p = synth.make_problem(cfg)
    lens = p.lengths
    el = np.uint16 if cfg.dtype == "bf16" else np.float32
    # The K-cache the slim step reads is banded (bands of 32 rows, head-major inside a band: SLIM_K_BANDED)
    # unless --k-layout rowmajor or a variant whose kernels read row-major caches only; the same step on the
    # row-major cache is timed beside it, and the vanilla kernel always reads row-major K and V.
    which = os.environ.get("SLIM_BENCH_STAGES") or (args.variant if args.variant != "auto" else binding.auto_variant_name(B, H, T, d, cfg.dtype))
    banded = args.k_layout == "banded" and which in ("fused", "fused_split")
    ts = (T + 31) // 32 * 32 if banded else T          # whole bands per sequence
    Kh = np.zeros((B, ts, d), dtype=el)
    Vh = np.zeros((B, ts, d), dtype=el)
    K64 = V64 = None
    for b, sq in enumerate(p.seqs):
        n = int(lens[b])
        Kb = synth.project_cache(sq.X, p.w.W_K)
        Vb = synth.project_cache(sq.X, p.w.W_V)
        Kh[b, :n] = synth.to_storage(Kb, cfg.dtype)
        Vh[b, :n] = synth.to_storage(Vb, cfg.dtype)
        if b == 0:
            K64, V64 = Kb, Vb          # the oracle's own fp64 caches for the CPU baseline
        sq.X = None
    wkv, rcond = binding.slim_prepare_wkv(p.w.W_K, p.w.W_V)
    log(f"[bench] inputs ready in {time.time() - t0:.1f} s (rcond(W_K) ~ {rcond:.2e})")

    to_device = binding.to_device
    k_bytes_alloc = Kh.nbytes
    ncopies = args.copies or max(2, int(np.ceil(512e6 / k_bytes_alloc)) + 1)
    Ks = [to_device(Kh) for _ in range(ncopies)]
    Vs = [to_device(Vh) for _ in range(ncopies)]
    Kbs = None
    if banded:
        Kbh = binding.slim_band_kcache(Kh, H)
        Kbs = [to_device(Kbh) for _ in range(ncopies)]
        del Kbh
    del Kh, Vh
    q = to_device(p.q.astype(np.float32))
    # W_KV rotates with the cache copies: at small batch it is a quarter of the step's bytes and one
    # buffer would be served by the memory-side cache
    w_host = binding.slim_pack_weights(wkv, cfg.dtype)
    wcopies = max(2, int(np.ceil(512e6 / w_host.nbytes)) + 1) if w_host.nbytes < 512e6 else 2
    wcopies = min(wcopies, 24)
    Wkvs = [to_device(w_host) for _ in range(wcopies)]
    lens_dev = torch.from_numpy(lens).cuda()
    out = torch.zeros((B, d), device="cuda", dtype=torch.float32)
    out_v = torch.zeros_like(out)
    ws = torch.empty(binding.slim_workspace_bytes(B, H, T, d, cfg.dtype), dtype=torch.uint8, device="cuda")
    ragged = bool((lens != T).any())
    kw = dict(dtype=cfg.dtype, workspace=ws, t_stride=ts)
    if ragged:
        kw.update(seq_lens=lens_dev, seq_lens_host=lens)
    rope_bytes = 0.0
    if args.rope:
        # vanilla keeps reading the same buffers: its cache would hold the rotated keys, same bytes
        kw_rope = dict(rope_table=to_device(binding.slim_rope_table(T, d_k, 10000.0)))
        rope_bytes = float(T) * (d_k // 2) * 8
    else:
        kw_rope = {}
    variant = {"auto": binding.VARIANT_AUTO, "generic": binding.VARIANT_GENERIC,
               "fused": binding.VARIANT_FUSED, "fused_split": binding.VARIANT_FUSED_SPLIT}[args.variant]
    binding.slim_init()

    def slim(i, variant=variant, **extra):
        if banded:
            binding.slim_decode(q, Kbs[i % ncopies], Wkvs[i % wcopies], out, B, H, T, d, variant=variant,
                                k_layout=binding.K_BANDED, **kw, **kw_rope, **extra)
        else:
            binding.slim_decode(q, Ks[i % ncopies], Wkvs[i % wcopies], out, B, H, T, d, variant=variant, **kw, **kw_rope, **extra)

    def slim_rowmajor(i):
        binding.slim_decode(q, Ks[i % ncopies], Wkvs[i % wcopies], out, B, H, T, d, variant=variant, **kw, **kw_rope)

    def vanilla(i, **extra):
        binding.vanilla_kv_decode(q, Ks[i % ncopies], Vs[i % ncopies], out_v, B, H, T, d, **kw, **extra)

    calibration_copy(args, torch)
    log("[bench] timing slim_decode ...")
    ms_slim = timed(torch, slim, args.steps, args.warmup)
    ms_slim_rowmajor = timed(torch, slim_rowmajor, args.steps, args.warmup) if (banded and not args.no_rowmajor_leg) else None
    log("[bench] timing vanilla_kv_decode ...")
    ms_van = timed(torch, vanilla, args.steps, args.warmup)
    # hot numbers (one buffer, may be served by the memory-side cache)
    ms_slim_hot = timed(torch, lambda i: slim(0), args.steps, 3)
    # the read rate this GPU sustains on the same buffers, same process: the practical ceiling of the K stream
    ms_probe = timed(torch, lambda i: binding.slim_read_probe(Ks[i % ncopies]), max(10, args.steps // 4), 3)
    probe_gbps = k_bytes_alloc / (ms_probe * 1e-3) / 1e9

    # per-kernel durations, HIP events on the launch stream (second pass over the same steps)
    log("[bench] per-kernel event timing ...")
    stage = binding.new_stage_buffer()
    acc = np.zeros(binding.MAX_STAGES)
    for i in range(args.steps):
        slim(i, stage_ms=stage)
        acc += np.array(list(stage))
    acc /= args.steps
    vstage = binding.new_stage_buffer()
    vacc = 0.0
    for i in range(args.steps):
        vanilla(i, stage_ms=vstage)
        vacc += vstage[0]
    vacc /= args.steps

    names = list(STAGES[which])
    k_bytes = float(lens.astype(np.int64).sum()) * d * es            # K-cache rows read once
    w_bytes = float(d) * d * es                                       # W_KV once per step
    one_launch = which == "fused" and acc[1] == 0.0                   # B <= 16: merge + projection inside
    split_ms = None
    if which == "fused":
        # the K stream alone (scores, softmax, weighted sum) and the merge + projection as launches of their own
        sacc = np.zeros(binding.MAX_STAGES)
        for i in range(args.steps):
            slim(i, variant=binding.VARIANT_FUSED_SPLIT, stage_ms=stage)
            sacc += np.array(list(stage))
        sacc /= args.steps
        split_ms = (float(sacc[0]), float(sacc[1]))
    if one_launch:
        names = ["fused_stream"]
    dom = int(np.argmax(acc[:len(names)]))
    alg_bytes = {"project": w_bytes, "project_mfma": w_bytes}.get(names[dom], k_bytes + rope_bytes + (w_bytes if one_launch else 0.0))
    kern_s = acc[dom] * 1e-3
    achieved = alg_bytes / kern_s / 1e9
    roofline = {"bound": "hbm", "kernel": names[dom] + (" (one launch: stream + merge + projection)" if one_launch else ""),
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": None if args.rope else measured_traffic(cfg.index, names[dom]),
                "algorithmic_bytes": alg_bytes, "kernel_ms": round(float(acc[dom]), 5),
                "stage_ms": {n: round(float(acc[i]), 5) for i, n in enumerate(names)}}

    cpu = None
    if with_cpu and not args.no_cpu_baseline:
        # the only place bench.py touches the oracle: it is timed as it stands, and its result
        # for sequence 0 is compared with what the timed GPU path produced
        from oracle import mha_oracle as orc
        log("[bench] timing the CPU oracle (decode step only, fp64 K and V resident) ...")
        n0 = int(lens[0])
        Kc, Vc = K64[:n0], V64[:n0]
        ref0 = orc.vanilla_decode_rope(p.q[0], Kc, Vc, H) if args.rope else orc.vanilla_decode(p.q[0], Kc, Vc, H)
        slim(0)
        torch.cuda.synchronize()
        got0 = out[0].cpu().numpy().astype(np.float64).reshape(H, d_k)
        r0 = ref0.reshape(H, d_k)
        err = float((np.abs(got0 - r0).max(axis=1) / np.abs(r0).max(axis=1)).max())
        reps, t_cpu0, c0 = 0, time.perf_counter(), os.times()
        while reps < 3 or (time.perf_counter() - t_cpu0 < 10.0 and reps < 200):
            orc.vanilla_decode(p.q[0], Kc, Vc, H)
            reps += 1
        wall = time.perf_counter() - t_cpu0
        c1 = os.times()
        busy = (c1.user - c0.user) + (c1.system - c0.system)
        cpu = {"value": round(reps / wall, 3), "unit": "tokens/s", "cores": max(1, int(round(busy / wall))),
               "kind": "oracle", "host_cores": os.cpu_count(),
               "sample": f"sequence 0 of config {cfg.index} ({n0} rows x {d}), {reps} repeats of the fp64 vanilla decode step",
               "gpu_max_rel_err_vs_oracle_seq0": float(f"{err:.3e}")}

    ms = ms_slim
    k_gbps = k_bytes / (ms * 1e-3) / 1e9
    result = {
        "metric": "decode tokens/s (one attention layer step, K-cache only) + effective K-cache GB/s vs vanilla K+V, 1 GPU",
        "value": round(B / (ms * 1e-3), 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{cfg.index}] {cfg.name}" + (" + rotary keys (RoPE option 1, raw keys cached)" if args.rope else ""),
                   "B": B, "H": H, "d": d, "d_k": d_k, "T": T,
                   "sum_len": int(lens.sum()), "variant": which,
                   "k_layout": "banded (32-row bands, head-major)" if banded else "row-major",
                   "k_cache_copies_rotated": ncopies, "w_kv_copies_rotated": wcopies},
        "k_cache_gbps": round(k_gbps, 1),
        "k_cache_frac_of_hbm_peak": round(k_gbps / HBM_PEAK_GBPS, 4),
        "measured_read_stream_gbps": round(probe_gbps, 1),
        "k_cache_frac_of_measured_stream_peak": round(k_gbps / probe_gbps, 4),
        "ms_per_step_hot_single_buffer": round(ms_slim_hot, 5),
        "vanilla_kv_ms_per_step": round(ms_van, 5), "vanilla_kv_kernel_ms": round(vacc, 5),
        "vanilla_kv_gbps": round(2 * k_bytes / (ms_van * 1e-3) / 1e9, 1),
        "speedup_vs_vanilla_kv": round(ms_van / ms, 3),
        "bytes_ratio_vanilla_over_slim": round(2 * k_bytes / (k_bytes + w_bytes), 3),
        "roofline": roofline, "cpu_baseline": cpu,
    }
    if ms_slim_rowmajor is not None:
        # the same step on the row-major cache [B][T][d]
        result["rowmajor_k_cache"] = {"ms_per_step": round(ms_slim_rowmajor, 5),
                                      "k_cache_gbps": round(k_bytes / (ms_slim_rowmajor * 1e-3) / 1e9, 1),
                                      "speedup_vs_vanilla_kv": round(ms_van / ms_slim_rowmajor, 3)}
    if split_ms is not None:
        # K1 + K2 (the K stream) apart from K3 (merge + W_KV projection), as two launches
        result["k_stream_only_ms"] = round(split_ms[0], 5)
        result["k_stream_only_gbps"] = round(k_bytes / (split_ms[0] * 1e-3) / 1e9, 1)
        result["k_stream_only_frac_of_hbm_peak"] = round(k_bytes / (split_ms[0] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
        result["merge_projection_ms"] = round(split_ms[1], 5)
    del Ks, Vs, Kbs, Wkvs, ws
    torch.cuda.empty_cache()
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=None, choices=[0, 1, 2, 3, 4],
                    help="time this config only (default: configs[2], the largest single-GPU one, as the headline, "
                         "with configs[1] nested in the same line)")
    ap.add_argument("--variant", default="auto", choices=["auto", "generic", "fused", "fused_split"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-rowmajor-leg", action="store_true",
                    help="with the banded layout: do not also time the step on the row-major cache (keeps a profile's per-kernel averages to one layout)")
    ap.add_argument("--k-layout", default="banded", choices=["banded", "rowmajor"],
                    help="layout of the K-cache slim_decode reads (the fast path only; vanilla_kv_decode reads row-major K and V)")
    ap.add_argument("--copies", type=int, default=0, help="K-cache copies to rotate over (0 = enough to exceed 512 MB)")
    ap.add_argument("--rope", action="store_true",
                    help="keys carry rotary positions: slim_decode rotates the raw cached keys for the scores (K-cache configs)")
    ap.add_argument("--ecache", action="store_true",
                    help="config 3 only: the cross-attention layer reads the encoder output E through slim_decode_xcache "
                         "(option 2 of the encoder-decoder section) instead of a cross K-cache")
    ap.add_argument("--layers", type=int, default=1,
                    help="with --ecache: this many decoder layers in a row on one shared encoder output (random values; per-layer times)")
    ap.add_argument("--block", action="store_true",
                    help="time the whole attention block (slim_attention_block vs vanilla_attention_block) instead of the decode step")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a few plain 128 MiB device copies (a kernel of known traffic, for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1")

    import torch
    from paper_2503_05840_amd import binding, synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    binding.load()
    headline = 2 if args.config is None else args.config
    cfg = synth.CONFIGS[headline]
    if args.ecache:
        if headline != 3:
            sys.exit("bench.py: --ecache applies to config 3 (the encoder-decoder cross-attention shape)")
        if args.layers > 1:
            return bench_ecache_layers(args, cfg, torch, binding, synth)
        cfg = synth.scaled(cfg, kind="xcache", name=cfg.name + " as E-cache (option 2)")
    if cfg.kind == "xcache":
        if args.rope or args.block:
            sys.exit("bench.py: --rope and --block apply to the K-cache configs (0-3)")
        return bench_xcache(args, cfg, torch, binding, synth)
    if args.block:
        return bench_block(args, cfg, torch, binding, synth)
    result = bench_kcache(args, cfg, torch, binding, synth, with_cpu=True)
    if args.config is None:
        # the 16k-context single-sequence config rides along in the same line (no second oracle timing)
        extra = bench_kcache(args, synth.CONFIGS[1], torch, binding, synth, with_cpu=False)
        keep = ("ms_per_step", "value", "k_cache_gbps", "k_cache_frac_of_hbm_peak", "k_cache_frac_of_measured_stream_peak",
                "measured_read_stream_gbps", "vanilla_kv_ms_per_step", "speedup_vs_vanilla_kv", "bytes_ratio_vanilla_over_slim",
                "k_stream_only_ms", "k_stream_only_frac_of_hbm_peak", "merge_projection_ms", "roofline", "config")
        result["other_configs"] = {"configs[1]": {k: extra[k] for k in keep if k in extra}}
        # and, GPU figures only (a few seconds each), the cross-attention batch and the X-cache config
        extra = bench_kcache(args, synth.CONFIGS[3], torch, binding, synth, with_cpu=False)
        result["other_configs"]["configs[3]"] = {k: extra[k] for k in keep if k in extra}
        saved, args.no_cpu_baseline = args.no_cpu_baseline, True
        extra = bench_xcache(args, synth.CONFIGS[4], torch, binding, synth, emit=False)
        args.no_cpu_baseline = saved
        result["other_configs"]["configs[4]"] = {k: extra[k] for k in ("ms_per_step", "value", "x_cache_gbps", "vanilla_kv_ms_per_step",
                                                                          "speedup_vs_vanilla_kv", "roofline", "config") if k in extra}
    result["paper_context"] = ("paper reports no measurement; analytical: up to 2x for long context (memory-bound), "
                               "Whisper B=64 1.8x (K-only) / 5.3x (E-cache)")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
