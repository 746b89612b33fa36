#!/usr/bin/env python3
"""Bench of KVPR's per-layer decode hot path on one MI355X.

A "step" is one decode of one OPT-shaped attention layer through the whole path at the scheduler-chosen
split l*: H2D of X[0:l*] and KV[l*:s] from the pinned host store, new-token q/k/v projection, recompute GEMM,
decode attention over s+1 positions, output projection, store-back.  The layer's activations and cache start
in pinned host memory (that is where the method keeps them; moving them is the method), weights and the
decode token's input are resident in HBM.

With no --model the run covers every configuration the metric is quoted on, in one process, and prints ONE
JSON line: the headline fields are those of the largest layer shape (OPT-30B shape, hidden 7168, batch 32,
context 1024); `configs` holds the OPT-6.7B shape (at l* and at l in {0, s/4, s/2, 3s/4, s}), the OPT-13B
shape, the OPT-30B context sweep at batch 16 (s in {512, 1024, 2048, 4096}), the 40-layer OPT-13B-shaped
stack generating 32 tokens greedily, and the column-by-column schedule with offloaded weights.  --steps /
--warmup apply to every per-layer timing.  With --model the run is that one layer shape.

Paper context (A100 + PCIe 4.0, whole models, not comparable): up to 35.8 % lower decode latency and 46.2 %
higher throughput than its baselines.
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

PEAK_MFMA_F16_TFLOPS = 2500.0   # MI355X dense fp16 MFMA
PEAK_HBM_GBPS = 8000.0          # MI355X HBM3E


def median(v):
    v = sorted(v)
    return v[len(v) // 2]


def cpu_baseline(layer, n_seq: int, llama: bool = False):
    """The oracle as it stands (numpy float64, full recompute of K/V then attention) on the first
    n_seq sequences of the same batch, timed on this machine's host cores."""
    if llama:
        from oracle import kvpr_llama_oracle as ko
    else:
        from oracle import kvpr_oracle as ko
    sub = dict(layer)
    sub["X"] = np.ascontiguousarray(layer["X"][:, :n_seq])
    sub["x_new"] = np.ascontiguousarray(layer["x_new"][:n_seq])
    s = sub["X"].shape[0]
    empty = np.zeros((0, n_seq, 2 * layer["h"]))
    t0 = time.perf_counter()
    r = ko.layer_decode(sub, s, kv_stored=empty)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    return r["o"], dt, min(threads, len(os.sched_getaffinity(0)))


def store_sizes(k, mode, b, h):
    """(dtype flags, bytes of X per cached position, bytes of KV per cached position) for --store-int4."""
    q = {"none": 0, "kv": k.KVPR_KV_INT4, "both": k.KVPR_STORE_INT4}[mode]
    x_bpp = b * (k.kvpr_int4_row_bytes(h) if q & k.KVPR_X_INT4 else 2 * h)
    kv_bpp = b * (k.kvpr_int4_row_bytes(2 * h) if q & k.KVPR_KV_INT4 else 4 * h)
    return q, x_bpp, kv_bpp


def run_stack(args):
    """Layer-pipelined decode of a whole OPT-shaped stack (default OPT-13B: 40 layers, batch 32,
    prompt 1024, 32 greedy tokens).  Weights are random-init on the GPU, every layer's X and KV
    live in the pinned host store, layer i+1's transfers are prefetched while layer i computes."""
    import torch
    import kvpr_inputs
    import paper_2411_17089_amd as k
    h, H, d = kvpr_inputs.SHAPES[args.model]
    llama = args.model.startswith("llama")
    b, s, L, gen = args.batch, args.seq, args.layers, args.gen
    ffn, vocab = (kvpr_inputs.LLAMA_FFN[args.model], 32000) if llama else (4 * h, 50272)
    cm = {"eq10": k.KVPR_COST_EQ10, "ns": k.KVPR_COST_NS, "row": k.KVPR_COST_ROW, "pipe": k.KVPR_COST_PIPE}[args.cost_model]
    torch.manual_seed(0)
    rnd = lambda shape, sc: (torch.randn(shape, device="cuda", dtype=torch.float32) * sc).half()
    t0 = time.perf_counter()
    qflags, x_bpp, kv_bpp = store_sizes(k, args.store_int4, b, h)
    also_pipe = cm == k.KVPR_COST_EQ10 and args.extension_chunks > 0
    ctx = k.kvpr_create(L, h, H, d, ffn, b, s + (2 if also_pipe else 1) * (gen + args.warmup) + 3, dtype=k.KVPR_F16 | qflags,
                        arch=k.KVPR_ARCH_LLAMA if llama else k.KVPR_ARCH_OPT)
    keep, ws = [], []
    for i in range(L):
        if llama:   # no biases, RMSNorm gains, w1 = [gate; up]
            t = dict(wqkv=rnd((3 * h, h), 0.02), wo=rnd((h, h), 0.02), ln1_g=1 + rnd((h,), 0.05), w1=rnd((2 * ffn, h), 0.02),
                     w2=rnd((h, ffn), 0.02), ln2_g=1 + rnd((h,), 0.05))
        else:
            t = dict(wqkv=rnd((3 * h, h), 0.02), bqkv=rnd((3 * h,), 0.01), wo=rnd((h, h), 0.02), bo=rnd((h,), 0.01),
                     ln1_g=1 + rnd((h,), 0.05), ln1_b=rnd((h,), 0.02), w1=rnd((ffn, h), 0.02), b1=rnd((ffn,), 0.01),
                     w2=rnd((h, ffn), 0.02), b2=rnd((h,), 0.01), ln2_g=1 + rnd((h,), 0.05), ln2_b=rnd((h,), 0.02))
        keep.append(t)
        ws.append(k.make_weights(**t))
        X = torch.randn((s, b, h), device="cuda", dtype=torch.float16)        # post-LN activations ~ N(0,1)
        k.kvpr_store_write(ctx, i, 0, s, X.cpu().numpy(), None)
        k.kvpr_store_prefill_kv(ctx, i, s, ws[i])
    w_lm, emb = rnd((vocab, h), 0.02), rnd((vocab, h), 1.0)
    setup_s = time.perf_counter() - t0
    prof = k.kvpr_profile(ctx, b, s)
    k.kvpr_set_profile(ctx, prof, cm, args.granularity)
    k.kvpr_set_adaptive(ctx, args.adaptive)
    x = rnd((b, h), 1.0)
    x_out = torch.empty_like(x)
    logits = torch.empty((b, vocab), dtype=torch.float32, device="cuda")
    tokens = torch.empty((b,), dtype=torch.int32, device="cuda")
    seq = s
    def one_token(seq, x):
        splits, _ = k.kvpr_decode_step(ctx, seq, ws, x, x_out, None)
        if not args.no_greedy:
            k.kvpr_greedy_next(x_out, w_lm, emb, b, h, vocab, logits, tokens, x)
        return splits
    for _ in range(args.warmup):
        one_token(seq, x)
        seq += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    all_splits = []
    host_s = 0.0
    for _ in range(gen):
        h0 = time.perf_counter()
        all_splits.append(one_token(seq, x)[0])
        host_s += time.perf_counter() - h0
        seq += 1
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # one more token with per-layer event timing (synchronises at the end; not part of the timed region)
    _, tim = k.kvpr_decode_step(ctx, seq, ws, x, x_out, None, timing=True)
    tmean = lambda name: float(np.mean([getattr(t, name) for t in tim[2:]]))
    breakdown = {n: tmean("ms_" + n) for n in ("act_copy", "kv_copy", "recompute", "proj", "attn", "out", "store", "total")}
    link_bytes = float(sum(x_bpp * l + kv_bpp * (s + args.warmup + i - l) for i, l in enumerate(all_splits)) * L)
    result = {
        "metric": "decode_tokens_per_s_layer_pipelined_stack", "value": b * gen / wall, "unit": "tokens/s",
        "n_gpus": 1, "steps": gen, "warmup": args.warmup, "ms_per_step": wall * 1e3 / gen, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic (random-init weights and N(0,1) activations generated on the GPU, seed 0)",
        "config": {"workload": f"{args.model}-shaped stack, {L} layers, hidden {h}, batch {b}, prompt {s}, {gen} greedy tokens, "
                               f"vocab {vocab}, X and KV of every layer in pinned host memory", "cost_model": args.cost_model,
                   "granularity": args.granularity, "splits_first_last": [all_splits[0], all_splits[-1]],
                   "store_int4": args.store_int4},
        "ms_per_layer": wall * 1e3 / gen / L,
        "h2d_GBps_sustained": link_bytes / wall / 1e9, "h2d_peak_GBps": prof.h2d_peak_bytes_per_s / 1e9,
        "h2d_frac_of_peak": link_bytes / wall / prof.h2d_peak_bytes_per_s,
        "profile": {"v_com_GBps": prof.h2d_bytes_per_s / 1e9, "v_gpu_TFLOPs": prof.gemm_flops_per_s / 1e12},
        "adaptive_alpha": args.adaptive,
        "profile_at_end": {"v_com_GBps": k.kvpr_get_profile(ctx).h2d_bytes_per_s / 1e9,
                           "v_gpu_TFLOPs": k.kvpr_get_profile(ctx).gemm_flops_per_s / 1e12},
        "breakdown_ms_per_layer": breakdown, "host_enqueue_ms_per_token": host_s * 1e3 / gen,
        "pinned_store_GiB": L * (s + (2 if also_pipe else 1) * (gen + args.warmup) + 3) * (x_bpp + kv_bpp) / 2 ** 30, "setup_s": setup_s,
    }
    if also_pipe:
        # extension, not the paper's objective: the steady-state cost form (a prefetching pipeline pays max(link, GPU) per
        # layer, so it recomputes until the GPU is as busy as the link); same context, the generation simply goes on
        seq += 1
        k.kvpr_set_profile(ctx, prof, k.KVPR_COST_PIPE, args.granularity)
        for _ in range(args.warmup):
            one_token(seq, x)
            seq += 1
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        pipe_splits = []
        for _ in range(gen):
            pipe_splits.append(one_token(seq, x)[0])
            seq += 1
        torch.cuda.synchronize()
        wall_p = time.perf_counter() - t0
        result["extension_steady_state_cost_form"] = {
            "tokens_per_s": b * gen / wall_p, "ms_per_layer": wall_p * 1e3 / gen / L, "splits_first_last": [pipe_splits[0], pipe_splits[-1]],
            "context_first_last": [seq - gen, seq - 1],
            "note": "KVPR_COST_PIPE = max(link time, recompute + rest of the layer's GPU work); not in the paper"}
    k.kvpr_destroy(ctx)
    del keep, ws, w_lm, emb, logits
    torch.cuda.empty_cache()
    return result


def run_columns(args):
    """Throughput-oriented mode (column-by-column schedule, weights offloaded too): every layer's weights
    are loaded once per token and used for --gpu-batches batches.  Reports tokens/s with the scheduler's
    split and, for reference, with l = 0 (no recomputation: transfer the whole cache)."""
    import torch
    import kvpr_inputs
    import paper_2411_17089_amd as k
    h, H, d = kvpr_inputs.SHAPES[args.model]
    llama = args.model.startswith("llama")
    b, s, L, nb, gen = args.batch, args.seq, args.layers, args.gpu_batches, args.gen
    ffn = kvpr_inputs.LLAMA_FFN[args.model] if llama else 4 * h
    S = L * nb
    cm = {"eq10": k.KVPR_COST_EQ10, "ns": k.KVPR_COST_NS, "row": k.KVPR_COST_ROW, "pipe": k.KVPR_COST_PIPE}[args.cost_model]
    rng = np.random.default_rng(0)
    torch.manual_seed(0)
    qflags, x_bpp, kv_bpp = store_sizes(k, args.store_int4, b, h)
    also_pipe = cm == k.KVPR_COST_EQ10 and args.extension_chunks > 0
    passes = (3 if also_pipe else 2) + (1 if getattr(args, "weight_pipeline_ablation", False) else 0)
    ctx = k.kvpr_create_offload(L, h, H, d, ffn, b, s + passes * (gen + args.warmup) + 2, nb, dtype=k.KVPR_F16 | qflags,
                                arch=k.KVPR_ARCH_LLAMA if llama else k.KVPR_ARCH_OPT)
    rh = lambda shape, sc: (rng.standard_normal(shape, dtype=np.float32) * np.float32(sc)).astype(np.float16)
    t0 = time.perf_counter()
    base = dict(wqkv=rh((3 * h, h), 0.02), bqkv=rh((3 * h,), 0.01), wo=rh((h, h), 0.02), bo=rh((h,), 0.01),
                ln1_g=(1 + rh((h,), 0.05)).astype(np.float16), ln1_b=rh((h,), 0.02), w1=rh((ffn, h), 0.02), b1=rh((ffn,), 0.01),
                w2=rh((h, ffn), 0.02), b2=rh((h,), 0.01), ln2_g=(1 + rh((h,), 0.05)).astype(np.float16), ln2_b=rh((h,), 0.02))
    if llama:   # no biases, RMSNorm gains only, w1 = [gate; up]
        base = dict(wqkv=base["wqkv"], wo=base["wo"], ln1_g=base["ln1_g"], ln2_g=base["ln2_g"], w1=rh((2 * ffn, h), 0.02), w2=base["w2"])
    dev_w = {n: torch.from_numpy(a).cuda() for n, a in base.items()}
    wdev = k.make_weights(**dev_w)
    for j in range(L):
        # one random parameter set, rolled by j rows per layer: distinct bytes per layer without 40 host-side draws
        lay = {n: (np.roll(a, j, axis=0) if a.ndim == 2 else a) for n, a in base.items()}
        lay = {n: np.ascontiguousarray(a) for n, a in lay.items()}
        k.kvpr_weights_write(ctx, j, k.make_weights(**lay))
        dw = k.make_weights(**{n: torch.from_numpy(a).cuda() for n, a in lay.items()}) if j else wdev
        for q in range(nb):
            X = torch.randn((s, b, h), device="cuda", dtype=torch.float16)
            k.kvpr_store_write(ctx, j * nb + q, 0, s, X.cpu().numpy(), None)
            k.kvpr_store_prefill_kv(ctx, j * nb + q, s, dw)
    setup_s = time.perf_counter() - t0
    prof = k.kvpr_profile(ctx, b, s)
    k.kvpr_set_profile(ctx, prof, cm, args.granularity)
    k.kvpr_set_adaptive(ctx, args.adaptive)
    if args.hidden_offload:
        k.kvpr_set_hidden_offload(ctx, True)      # Algorithm 1's load_activation / store_activation of the layer inputs
    x = (torch.randn((nb, b, h), device="cuda") * 1.0).half()
    x_out = torch.empty_like(x)
    seq = s
    results = {}
    runs = [("kvpr", None), ("no_recompute", [0] * S)]
    if getattr(args, "weight_pipeline_ablation", False):
        runs.append(("kvpr_without_weight_pipeline", None))   # Table 2's "without hiding" arm: recompute waits for the whole layer
    if also_pipe:
        runs.append(("steady_state_cost_form", None))     # extension, not the paper's objective: see run_stack
    for name, splits in runs:
        k.kvpr_set_weight_pipeline(ctx, name != "kvpr_without_weight_pipeline")
        if name == "steady_state_cost_form":
            k.kvpr_set_profile(ctx, prof, k.KVPR_COST_PIPE, args.granularity)
        for _ in range(args.warmup):
            k.kvpr_decode_step_columns(ctx, seq, S, x, x_out, splits)
            seq += 1
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(gen):
            used, _ = k.kvpr_decode_step_columns(ctx, seq, S, x, x_out, splits)
            seq += 1
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        results[name] = {"tokens_per_s": nb * b * gen / wall, "ms_per_token_step": wall * 1e3 / gen,
                         "ms_per_layer_batch": wall * 1e3 / gen / S, "split": used[0]}
    blob_bytes = (4 * h * h + (3 if llama else 2) * ffn * h) * 2
    r = results["kvpr"]
    out = {
        "metric": "decode_tokens_per_s_column_schedule_weights_offloaded", "value": r["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": gen, "warmup": args.warmup, "ms_per_step": r["ms_per_token_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic (seeded random weights and N(0,1) activations; cache = GPU prefill)",
        "config": {"workload": f"{args.model}-shaped stack, {L} layers, {nb} GPU batches x batch {b} (effective batch {nb * b}), "
                               f"context {s}, {gen} tokens, weights ({blob_bytes / 2**20:.0f} MiB/layer), X and KV in pinned host memory",
                   "cost_model": args.cost_model, "granularity": args.granularity, "store_int4": args.store_int4},
        "kvpr": r, "no_recompute": results["no_recompute"],
        **({"kvpr_without_weight_pipeline": results["kvpr_without_weight_pipeline"]} if "kvpr_without_weight_pipeline" in results else {}),
        "speedup_over_no_recompute": results["no_recompute"]["ms_per_token_step"] / r["ms_per_token_step"],
        "profile": {"v_com_GBps": prof.h2d_bytes_per_s / 1e9, "v_gpu_TFLOPs": prof.gemm_flops_per_s / 1e12},
        "pinned_GiB": (S * (s + passes * (gen + args.warmup) + 2) * (x_bpp + kv_bpp) + L * blob_bytes) / 2 ** 30, "setup_s": setup_s,
    }
    if also_pipe:
        out["extension_steady_state_cost_form"] = dict(results["steady_state_cost_form"],
            note="KVPR_COST_PIPE = max(link time, recompute + rest of the layer's GPU work); not in the paper")
    k.kvpr_destroy(ctx)
    del dev_w, wdev
    torch.cuda.empty_cache()
    return out


def run_power_probe(args):
    """Evidence for what bounds the recompute GEMM on real data: shader clock and socket power (amd-smi, sampled twice a
    second from a side thread) while (a) the recompute GEMM of the OPT-6.7B shape and (b) a register-only loop of the
    same MFMA run for a few seconds each, on N(0,1) / N(0,0.02) operands, on a constant and on zeros."""
    import subprocess
    import threading
    import ctypes as C
    import torch
    import kvpr_inputs
    import paper_2411_17089_amd as k
    h, H, d = kvpr_inputs.SHAPES[args.model]
    b = args.batch
    split = args.split if args.split >= 0 else 832
    M = split * b
    A = torch.empty((M, h), device="cuda", dtype=torch.float16)
    W = torch.empty((2 * h, h), device="cuda", dtype=torch.float16)
    Cc = torch.empty((M, 2 * h), device="cuda", dtype=torch.float16)
    sink = torch.empty((256 * 512,), device="cuda", dtype=torch.float32)
    k.lib.kvpr_debug_mfma_loop.restype = C.c_int
    k.lib.kvpr_debug_mfma_loop.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int, C.c_void_p]
    stream = torch.cuda.current_stream().cuda_stream

    def find(obj, want):
        """first numeric 'value' under a key whose name contains `want` in amd-smi's JSON"""
        if isinstance(obj, dict):
            for key, v in obj.items():
                if want in key.lower():
                    if isinstance(v, dict) and "value" in v and isinstance(v["value"], (int, float)):
                        return float(v["value"])
                    if isinstance(v, dict) and "clk" in v:
                        r = find({"clk_": v["clk"]}, "clk_")
                        if r is not None:
                            return r
                    if isinstance(v, (int, float)):
                        return float(v)
                r = find(v, want)
                if r is not None:
                    return r
        elif isinstance(obj, list):
            for v in obj:
                r = find(v, want)
                if r is not None:
                    return r
        return None

    samples, stop, raw = [], threading.Event(), []
    def sampler():
        while not stop.is_set():
            try:
                txt = subprocess.run(["amd-smi", "metric", "-g", "0", "--clock", "--power", "--json"], capture_output=True,
                                     text=True, timeout=10).stdout
                j = json.loads(txt)
                if not raw:
                    raw.append(txt[:1500])
                samples.append((time.perf_counter(), find(j, "gfx_0"), find(j, "socket_power")))
            except Exception as e:   # amd-smi missing or not permitted: the rates are still reported
                if not raw:
                    raw.append("amd-smi failed: %r" % (e,))
            stop.wait(0.5)

    def sustained(fn, work, seconds):
        fn()
        torch.cuda.synchronize()
        n, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            for _ in range(20):
                fn()
            torch.cuda.synchronize()
            n += 20
        dt = time.perf_counter() - t0
        mine = [s for s in samples if s[0] >= t0 + 1.0 and s[0] <= t0 + dt]    # skip the first second (ramp)
        clk = [s[1] for s in mine if s[1] is not None]
        pw = [s[2] for s in mine if s[2] is not None]
        return {"TFLOPs": work * n / dt / 1e12, "seconds": dt, "launches": n, "samples": len(mine),
                "shader_clock_MHz_min_mean_max": [min(clk), sum(clk) / len(clk), max(clk)] if clk else None,
                "socket_power_W_min_mean_max": [min(pw), sum(pw) / len(pw), max(pw)] if pw else None}

    th = threading.Thread(target=sampler, daemon=True)
    th.start()
    out = {"shape": {"M": M, "N": 2 * h, "K": h}, "modes": {}}
    loop_iters = 4000
    for mode in ("normal", "constant", "zeros"):
        if mode == "normal":
            A.normal_()
            W.normal_()
            W.mul_(0.02)
        elif mode == "constant":
            A.fill_(0.5)
            W.fill_(0.015625)
        else:
            A.zero_()
            W.zero_()
        torch.cuda.synchronize()
        time.sleep(1.0)
        g = sustained(lambda: k.kvpr_recompute_gemm(A, W, None, Cc, M, 2 * h, h, 2 * h), 4.0 * M * h * h, args.probe_seconds)
        time.sleep(1.0)
        r = sustained(lambda: k.lib.kvpr_debug_mfma_loop(A.data_ptr(), W.data_ptr(), A.numel(), W.numel(), sink.data_ptr(), loop_iters, stream),
                      256.0 * 8 * loop_iters * 16 * 2 * 32 * 32 * 16, args.probe_seconds)
        out["modes"][mode] = {"recompute_gemm": g, "register_only_mfma_loop": r}
    stop.set()
    th.join(timeout=15)
    out["amd_smi_first_sample"] = raw[0] if raw else None
    print(json.dumps(out))


def run_kernels(args):
    """Standalone launches of the path's kernels at the bench shape, for rocprofv3 counter runs:
    a plain device copy of known size (reference for scaling FETCH_SIZE / WRITE_SIZE), the recompute
    GEMM at M = split*batch, decode attention over seq+1 positions, and the four token GEMMs of a decoder layer."""
    import torch
    import kvpr_inputs
    import paper_2411_17089_amd as k
    h, H, d = kvpr_inputs.SHAPES[args.model]
    b, s = args.batch, args.seq
    split = args.split if args.split >= 0 else 832
    torch.manual_seed(0)
    M = split * b
    A = torch.randn((M, h), device="cuda", dtype=torch.float16)
    W = (torch.randn((3 * h, h), device="cuda") * 0.02).half()
    bias = (torch.randn((3 * h,), device="cuda") * 0.01).half()
    kv = torch.empty((s + 1, b, 2 * h), device="cuda", dtype=torch.float16)
    kv.normal_()
    q = torch.randn((b, h), device="cuda", dtype=torch.float32)
    z = torch.empty((b, h), device="cuda", dtype=torch.float16)
    x = torch.randn((b, h), device="cuda", dtype=torch.float16)
    y16 = torch.empty((b, 2 * h), device="cuda", dtype=torch.float16)
    ws = torch.empty(k.kvpr_attention_workspace_bytes(b, h, H, s + 1), dtype=torch.uint8, device="cuda")
    src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    src.fill_(1)
    dst = torch.empty_like(src)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    out = {}
    def timed(name, fn):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(args.steps):
            e0, e1 = ev(), ev()
            e0.record(); fn(); e1.record(); e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        out[name] = median(ts)
    timed("copy_512MiB_ms", lambda: dst.copy_(src))
    timed("recompute_gemm_ms", lambda: k.kvpr_recompute_gemm(A, W[h:], bias[h:], kv, M, 2 * h, h, 2 * h))
    timed("attention_ms", lambda: k.kvpr_decode_attention(q, kv, z, ws, s + 1, b, h, H))
    # the four token GEMMs of a decoder layer as a context launches them (with its K-slice workspace)
    W4 = (torch.randn((4 * h, h), device="cuda") * 0.02).half()
    x4 = torch.randn((b, 4 * h), device="cuda", dtype=torch.float16)
    y4 = torch.empty((b, 4 * h), device="cuda", dtype=torch.float16)
    tws_bytes = k.kvpr_token_gemm_workspace_bytes(b, h)
    tws = torch.zeros(tws_bytes, dtype=torch.uint8, device="cuda")
    timed("token_gemm_qkv_ms", lambda: k.kvpr_token_gemm_ws(x, W, bias, q, y16, b, 3 * h, h, h, 2 * h, tws, tws_bytes))
    timed("token_gemm_out_ms", lambda: k.kvpr_token_gemm_ws(x, W, bias, None, y16, b, h, h, 0, h, tws, tws_bytes))
    timed("token_gemm_ffn_up_ms", lambda: k.kvpr_token_gemm_ws(x, W4, None, None, y4, b, 4 * h, h, 0, 4 * h, tws, tws_bytes))
    timed("token_gemm_ffn_down_ms", lambda: k.kvpr_token_gemm_ws(x4, W4, None, None, y16, b, h, 4 * h, 0, h, tws, tws_bytes))
    for name, n_w in (("qkv", 3), ("out", 1), ("ffn_up", 4), ("ffn_down", 4)):
        out[f"token_gemm_{name}_GBps"] = n_w * h * h * 2 / out[f"token_gemm_{name}_ms"] / 1e6
    out["recompute_gemm_TFLOPs"] = 4.0 * M * h * h / out["recompute_gemm_ms"] / 1e9
    out["attention_GBps"] = 2.0 * b * (s + 1) * h * 2 / out["attention_ms"] / 1e6
    out["shape"] = {"model": args.model, "batch": b, "seq": s, "split": split, "M": M, "N": 2 * h, "K": h}
    print(json.dumps(out))


def profile_figures(model, b, s):
    """Figures that only a profiler run can give (rocprofv3 counter runs of `bench.py --kernels`, committed under
    profiles/): HBM-side bytes per recomputed position and the fraction of cycles the MFMA unit was busy."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    return json.load(open(path)).get(f"recompute_gemm/{model}/b{b}/s{s}")


def run_layer(args, model, b, s, split_arg=-1, sweep=(), attention=True, extension=False, cpu=False):
    """One attention layer of `model` shape at batch b, context s: profile, plan, calibrate, warm up, time
    args.steps decodes.  Returns the figures of the case as a dict."""
    import torch
    import kvpr_inputs
    import paper_2411_17089_amd as k
    h, H, d = kvpr_inputs.SHAPES[model]
    cm = {"eq10": k.KVPR_COST_EQ10, "ns": k.KVPR_COST_NS, "row": k.KVPR_COST_ROW, "pipe": k.KVPR_COST_PIPE}[args.cost_model]

    layer = kvpr_inputs.make_layer(0, b, s, h, H)
    f16 = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    llama = model.startswith("llama")
    arch = k.KVPR_ARCH_LLAMA if llama else k.KVPR_ARCH_OPT
    wqkv = f16(np.concatenate([layer["Wq"].T, layer["Wk"].T, layer["Wv"].T], 0))
    bqkv = f16(np.concatenate([layer["bq"], layer["bk"], layer["bv"]]))
    wo, bo, x_new = f16(layer["Wo"].T), f16(layer["bo"]), f16(layer["x_new"])
    w = k.make_weights(wqkv=wqkv, wo=wo) if llama else k.make_weights(wqkv=wqkv, bqkv=bqkv, wo=wo, bo=bo)
    out = torch.empty((b, h), dtype=torch.float16, device="cuda")

    # bytes per cached position (whole batch) as they cross the link, flops per recomputed position (Eq. 6, Eq. 8)
    qflags, x_bpp, kv_bpp = store_sizes(k, args.store_int4, b, h)
    f_pp = 4 * b * h * h
    ctx = k.kvpr_create(1, h, H, d, 0, b, s + 2, dtype=k.KVPR_F16 | qflags, arch=arch)
    k.kvpr_store_write(ctx, 0, 0, s, layer["X"], None)
    k.kvpr_store_prefill_kv(ctx, 0, s, w)          # stand-in for prefill: cache = X.[Wk|Wv]+b, computed on the GPU

    k.kvpr_set_keep_warm(ctx, args.keep_warm)
    prof_sustained = k.kvpr_profile(ctx, b, s)
    # one layer at a time with an idle GPU in between: v_gpu as such a step runs the GEMM (rehearsed at the planned split)
    prof0 = k.kvpr_profile_step(ctx, b, s, prof_sustained)
    k.kvpr_set_profile(ctx, prof0, cm, args.granularity)
    k.kvpr_set_chunks(ctx, args.chunks)
    # Refine the two constants: a few untimed decodes at the planned split, each timed by its own events and waited
    # for; the link rate and the GEMM rate (flops as the cost model charges them) are the medians over these decodes.
    # Medians, not the library's moving average (kvpr_set_adaptive): the first decodes on a fresh store find its pages
    # still in the CPU's caches and single copies run at 30-45 GB/s, which a six-sample moving average does not forget.
    prof = prof0
    trace = []
    if args.calibrate > 0 and split_arg < 0:
        l_cal, _ = k.kvpr_plan_split_linear(prof0, cm, args.chunks if cm == k.KVPR_COST_EQ10 else 1, s, x_bpp, kv_bpp, f_pp, args.granularity)
        for _ in range(2):
            k.kvpr_layer_decode(ctx, 0, s, l_cal, w, x_new, out)
            torch.cuda.synchronize()
        for i in range(args.calibrate):
            k.kvpr_layer_decode_timed(ctx, 0, s, l_cal, w, x_new, out, i)
            torch.cuda.synchronize()
            t = k.kvpr_timing_read(ctx, i)
            trace.append([t.ms_act_copy + t.ms_kv_copy, t.ms_recompute])
        prof = k.kvpr_profile_t.from_buffer_copy(prof0)
        link_ms = float(np.median([t[0] for t in trace]))
        gemm_ms = float(np.median([t[1] for t in trace]))
        if link_ms > 0:
            prof.h2d_bytes_per_s = (x_bpp * l_cal + kv_bpp * (s - l_cal)) / (link_ms * 1e-3)
        if l_cal > 0 and gemm_ms > 0 and args.chunks == 1:
            flops = f_pp * l_cal
            if prof0.gemm_round_flops > 0:
                flops = -(-flops // prof0.gemm_round_flops) * prof0.gemm_round_flops
            prof.gemm_flops_per_s = flops / (gemm_ms * 1e-3)
        k.kvpr_set_profile(ctx, prof, cm, args.granularity)
        trace = [[round(a, 3), round(g, 3)] for a, g in trace]
    pchunks = args.chunks if cm == k.KVPR_COST_EQ10 else 1
    # The split comes from the calibrated constants.  Every "bound" below is a cost model evaluated with the start-up
    # profile's constants (isolated copy rate, GEMM under a concurrent copy), so no ratio is measured against itself:
    #   builder's bound: the cost form in use with l restricted to multiples of the granularity and the GEMM charged
    #                    in whole rounds of one tile per compute unit;
    #   plain Eq. 10:    the paper's form as printed, every integer l, divisible GEMM work.
    l_star, _ = k.kvpr_plan_split_linear(prof, cm, pchunks, s, x_bpp, kv_bpp, f_pp, args.granularity)
    l_uncal, _ = k.kvpr_plan_split_linear(prof0, cm, pchunks, s, x_bpp, kv_bpp, f_pp, args.granularity)
    plain = k.kvpr_profile_t.from_buffer_copy(prof0)
    plain.gemm_round_flops = 0
    plain.h2d_latency_s = plain.gemm_latency_s = 0.0
    l_plain, t_plain = k.kvpr_plan_split_linear(plain, k.KVPR_COST_EQ10, 1, s, x_bpp, kv_bpp, f_pp, 1)
    l_eq10, t_eq10 = k.kvpr_plan_split_linear(prof0, k.KVPR_COST_EQ10, 1, s, x_bpp, kv_bpp, f_pp, args.granularity)

    def timed_at(split, steps):
        # warm-up through the same entry point, timing slots and queue depth as the timed decodes: the runtime grows its
        # pools (completion signals, timing events) the first time that many operations are in flight at once, and
        # while it does, running copies and kernels take up to twice as long
        for i in range(args.warmup):
            k.kvpr_layer_decode_timed(ctx, 0, s, split, w, x_new, out, i % steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            k.kvpr_layer_decode_timed(ctx, 0, s, split, w, x_new, out, i)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return wall * 1e3 / steps, [k.kvpr_timing_read(ctx, i) for i in range(steps)]

    split = l_star if split_arg < 0 else split_arg
    t_bound_split = k.kvpr_cost_linear(prof0, cm, pchunks, split, s, x_bpp, kv_bpp, f_pp)
    t_plain_split = k.kvpr_cost_linear(plain, k.KVPR_COST_EQ10, 1, split, s, x_bpp, kv_bpp, f_pp)
    ms_step, tim = timed_at(split, args.steps)

    mean = lambda name: float(np.mean([getattr(t, name) for t in tim]))
    median = lambda name: float(np.median([getattr(t, name) for t in tim]))
    ms_gemm, ms_attn = mean("ms_recompute"), mean("ms_attn")
    ms_act, ms_kv = mean("ms_act_copy"), mean("ms_kv_copy")
    gemm_flops = 4.0 * b * split * h * h
    attn_bytes = 2.0 * b * (s + 1) * h * 2
    # ms_attn sums the two attention phases; with a packed cache the transferred rows are read in packed form
    attn_phase_bytes = float(2 * b * (split + 1) * h * 2 + kv_bpp * (s - split)) if qflags & k.KVPR_KV_INT4 else attn_bytes
    two_phase = bool(qflags & k.KVPR_KV_INT4 or split >= 128)
    attn_kernel = "attention_partial_ranged x2 (+combine)" if two_phase else "attention_partial (+combine)"
    h2d_bytes = float(x_bpp * split + kv_bpp * (s - split))
    gemm_tflops = gemm_flops / (ms_gemm * 1e-3) / 1e12 if split > 0 else 0.0
    attn_gbps = attn_phase_bytes / (ms_attn * 1e-3) / 1e9
    h2d_gbps = h2d_bytes / ((ms_act + ms_kv) * 1e-3) / 1e9

    res = {
        "workload": f"{model}-shaped attention layer, hidden {h}, {H} heads x {d}, batch {b}, context {s}, "
                    f"decode 1 token at split l={split}",
        "model": model, "batch": b, "context": s, "split": split, "l_star": l_star,
        "l_star_from_startup_profile_alone": l_uncal,
        "ms_per_layer": ms_step, "tokens_per_s": b / (ms_step * 1e-3),
        "ms_assemble": mean("ms_assemble"), "ms_total_events": mean("ms_total"),
        # per-step spread (event time first enqueue -> end of the step): the link of these boxes has occasional slow stretches
        "ms_total_events_min_median_max": [float(np.min([t.ms_total for t in tim])), float(np.median([t.ms_total for t in tim])),
                                           float(np.max([t.ms_total for t in tim]))],
        "bounds": {
            "which": "builder = cost form '%s', l a multiple of %d, GEMM charged in whole 256-tile rounds; plain = Eq. 10 as "
                     "printed (every integer l, divisible work); both with the start-up profile's constants" % (args.cost_model, args.granularity),
            "builder_bound_ms_at_split": t_bound_split * 1e3,
            "builder_eq10_bound_ms_at_its_optimum": t_eq10 * 1e3, "builder_eq10_l_star": l_eq10,
            "plain_eq10_bound_ms_at_split": t_plain_split * 1e3,
            "plain_eq10_bound_ms_at_its_optimum": t_plain * 1e3, "plain_eq10_l_star": l_plain,
            "assemble_over_builder_bound": mean("ms_assemble") / (t_bound_split * 1e3),
            "assemble_over_plain_eq10_at_split": mean("ms_assemble") / (t_plain_split * 1e3),
            "assemble_over_plain_eq10_optimum": mean("ms_assemble") / (t_plain * 1e3),
            "step_over_builder_bound": ms_step / (t_bound_split * 1e3),
            "step_over_plain_eq10_optimum": ms_step / (t_plain * 1e3),
        },
        "breakdown_ms": {"act_copy": ms_act, "kv_copy": ms_kv, "recompute": ms_gemm, "proj": mean("ms_proj"),
                         "attn": ms_attn, "out": mean("ms_out"), "store": mean("ms_store"), "attn_early": mean("ms_attn_early")},
        "profile": {"v_com_GBps": prof.h2d_bytes_per_s / 1e9, "v_gpu_TFLOPs": prof.gemm_flops_per_s / 1e12,
                    "before_calibration": {"v_com_GBps": prof0.h2d_bytes_per_s / 1e9, "v_gpu_TFLOPs": prof0.gemm_flops_per_s / 1e12,
                                           "v_gpu_back_to_back_under_copy_TFLOPs": prof_sustained.gemm_flops_per_s / 1e12},
                    "calibration_decodes": args.calibrate if split_arg < 0 else 0,
                    "calibration_split": l_cal if trace else None, "calibration_link_ms_gemm_ms": trace,
                    "v_gpu_alone_TFLOPs": prof.gemm_alone_flops_per_s / 1e12, "h2d_peak_GBps": prof.h2d_peak_bytes_per_s / 1e9,
                    "d2h_GBps": prof.d2h_bytes_per_s / 1e9, "attn_GBps": prof.attn_bytes_per_s / 1e9},
        # means over the timed steps (what rocprofv3's average shows) and, beside them, medians: a step that a host
        # preemption or a stalled copy stretches also finds the GPU at idle clocks for its GEMM
        "gemm": {"TFLOPs": gemm_tflops, "frac_of_mfma_peak": gemm_tflops / PEAK_MFMA_F16_TFLOPS, "avg_ms": ms_gemm,
                 "flops_per_launch": gemm_flops, "median_ms": median("ms_recompute"),
                 "median_TFLOPs": gemm_flops / (median("ms_recompute") * 1e-3) / 1e12 if split > 0 else 0.0},
        "h2d": {"achieved_GBps": h2d_gbps, "measured_pinned_peak_GBps": prof.h2d_peak_bytes_per_s / 1e9,
                "frac": h2d_gbps / (prof.h2d_peak_bytes_per_s / 1e9), "bytes_per_step": h2d_bytes,
                "median_GBps": h2d_bytes / (float(np.median([t.ms_act_copy + t.ms_kv_copy for t in tim])) * 1e-3) / 1e9},
        "attention_in_layer_event_pairs": {"kernels": attn_kernel, "ms": ms_attn, "ms_before_cache_fence": mean("ms_attn_early"),
                                           "bytes": attn_phase_bytes, "GBps": attn_gbps,
                                           "note": "event pairs around single 20-90 us launches carry ~10 us of gap each"},
    }

    if args.keep_warm > 0 and split > 0:
        # the same split without the clock keep-alive: the GEMM then starts on a GPU that idled through the activation copy
        k.kvpr_set_keep_warm(ctx, 0.0)
        ms_cold, tim_cold = timed_at(split, args.steps)
        k.kvpr_set_keep_warm(ctx, args.keep_warm)
        ms_gemm_cold = float(np.mean([t.ms_recompute for t in tim_cold]))
        res["without_keep_warm"] = {"ms_per_layer": ms_cold, "gemm_avg_ms": ms_gemm_cold,
                                    "gemm_TFLOPs": gemm_flops / (ms_gemm_cold * 1e-3) / 1e12,
                                    "ms_assemble": float(np.mean([t.ms_assemble for t in tim_cold]))}
        res["keep_warm_fraction"] = args.keep_warm

    if attention:
        # the attention exactly as the layer runs it at this split (two ranged launches + combine when l >= 128, one
        # launch otherwise) and the single-launch kernel, each 20 times back to back between one pair of events
        kv_res = torch.randn((s + 1, b, 2 * h), dtype=torch.float16, device="cuda")
        q_res = torch.randn((b, h), dtype=torch.float32, device="cuda")
        z_res = torch.empty((b, h), dtype=torch.float16, device="cuda")
        ws_res = torch.empty(k.kvpr_attention_workspace_bytes(b, h, H, s + 1), dtype=torch.uint8, device="cuda")
        def b2b(fn):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                fn()
            e1.record()
            e1.synchronize()
            return e0.elapsed_time(e1) / 20
        ms_single = b2b(lambda: k.kvpr_decode_attention(q_res, kv_res, z_res, ws_res, s + 1, b, h, H))
        ms_layer_form = (b2b(lambda: k.kvpr_decode_attention_mixed(q_res, kv_res, None, z_res, ws_res, s + 1, split, b, h, H))
                         if two_phase and not qflags else ms_single)
        del kv_res
        res["attention"] = {
            "as_in_layer": {"kernels": attn_kernel if not qflags else "attention_partial (+combine)", "avg_ms": ms_layer_form,
                            "GBps": attn_bytes / (ms_layer_form * 1e-3) / 1e9,
                            "frac_of_hbm_peak": attn_bytes / (ms_layer_form * 1e-3) / 1e9 / PEAK_HBM_GBPS},
            "single_launch": {"kernels": "attention_partial (+combine)", "avg_ms": ms_single,
                              "GBps": attn_bytes / (ms_single * 1e-3) / 1e9,
                              "frac_of_hbm_peak": attn_bytes / (ms_single * 1e-3) / 1e9 / PEAK_HBM_GBPS},
            "bytes_per_launch": attn_bytes,
        }

    if sweep:
        res["split_sweep"] = []
        for l in sweep:
            ms_l, tim_l = timed_at(l, args.steps)
            t_b = k.kvpr_cost_linear(prof0, cm, pchunks, l, s, x_bpp, kv_bpp, f_pp)
            t_p = k.kvpr_cost_linear(plain, k.KVPR_COST_EQ10, 1, l, s, x_bpp, kv_bpp, f_pp)
            asm = float(np.mean([t.ms_assemble for t in tim_l]))
            res["split_sweep"].append({"split": l, "ms_per_layer": ms_l, "ms_assemble": asm,
                                       "assemble_over_builder_bound": asm / (t_b * 1e3), "assemble_over_plain_eq10": asm / (t_p * 1e3)})
        k.kvpr_layer_decode(ctx, 0, s, split, w, x_new, out)      # leave `out` at the headline split for the oracle check
        torch.cuda.synchronize()

    if extension and args.extension_chunks > 1 and args.chunks == 1 and cm == k.KVPR_COST_EQ10 and split_arg < 0:
        # same layer, same number of steps, X[0:l] copied in parts with each part's GEMM started as it lands
        c = args.extension_chunks
        k.kvpr_set_chunks(ctx, c)
        l_c, _ = k.kvpr_plan_split_linear(prof, k.KVPR_COST_EQ10, c, s, x_bpp, kv_bpp, f_pp, args.granularity)
        t_c = k.kvpr_cost_linear(prof0, k.KVPR_COST_EQ10, c, l_c, s, x_bpp, kv_bpp, f_pp)
        for _ in range(args.warmup):
            k.kvpr_layer_decode(ctx, 0, s, l_c, w, x_new, out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            k.kvpr_layer_decode(ctx, 0, s, l_c, w, x_new, out)
        torch.cuda.synchronize()
        ms_c = (time.perf_counter() - t0) * 1e3 / args.steps
        k.kvpr_set_chunks(ctx, 1)
        res["extension_chunked_copy"] = {
            "chunks": c, "l_star": l_c, "ms_per_layer": ms_c, "tokens_per_s": b / (ms_c * 1e-3),
            "chunked_model_bound_ms": t_c * 1e3, "step_over_chunked_bound": ms_c / (t_c * 1e3),
            "step_over_plain_eq10_optimum": ms_c / (t_plain * 1e3), "speedup_over_paper_schedule": ms_step / ms_c,
            "note": "not the paper's schedule: X[0:l] travels in parts and each part is recomputed as it lands; "
                    "same outputs bit for bit"}

    if cpu:
        n_seq = min(args.cpu_seqs, b)
        o_ref, dt, cores = cpu_baseline(layer, n_seq, llama)
        got = out.float().cpu().numpy()[:n_seq]
        res["cpu_baseline"] = {
            "value": n_seq / dt, "unit": "tokens/s per layer", "cores": cores, "kind": "oracle",
            "sample": f"{model} shape, batch {b}, context {s}: first {n_seq} of the {b} sequences of the layer, one decode step: numpy "
                      f"float64 recompute of all {s} K/V rows (Eq. 1) + attention + output projection; {dt:.2f} s",
            ("max_rel_err_gpu_vs_oracle_on_sample" if not qflags else "max_rel_err_gpu_over_4bit_store_vs_exact_oracle_on_sample"):
                float(np.max(np.abs(got - o_ref)) / np.max(np.abs(o_ref))),
        }
    k.kvpr_destroy(ctx)
    del wqkv, wo, layer
    torch.cuda.empty_cache()
    return res


def mfma_ceiling(seconds=1.5):
    """What this box's power management lets the fp16 MFMA unit sustain on this kind of data: a register-only loop of the
    GEMM's instruction (no LDS, no global traffic after the first loads) on N(0,1) x N(0,0.02) operands, in launches of
    about the GEMM's length, back to back for `seconds` after a second of ramp."""
    import ctypes as C
    import torch
    import paper_2411_17089_amd as k
    k.lib.kvpr_debug_mfma_loop.restype = C.c_int
    k.lib.kvpr_debug_mfma_loop.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int, C.c_void_p]
    g = torch.Generator(device="cuda").manual_seed(0)
    a = torch.randn((1 << 22,), device="cuda", dtype=torch.float32, generator=g).half()
    w = (torch.randn((1 << 22,), device="cuda", dtype=torch.float32, generator=g) * 0.02).half()
    sink = torch.empty((256 * 512,), device="cuda", dtype=torch.float32)
    stream = torch.cuda.current_stream().cuda_stream
    iters = 6000
    flops = 256 * 8 * iters * 16 * 32768.0
    def launch():
        rc = k.lib.kvpr_debug_mfma_loop(a.data_ptr(), w.data_ptr(), a.numel(), w.numel(), sink.data_ptr(), iters, stream)
        if rc != 0:
            raise RuntimeError("kvpr_debug_mfma_loop failed: %d" % rc)
    t_end = time.perf_counter() + 1.0
    while time.perf_counter() < t_end:
        for _ in range(10):
            launch()
        torch.cuda.synchronize()
    n, t0 = 0, time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(10):
            launch()
        torch.cuda.synchronize()
        n += 10
    dt = time.perf_counter() - t0
    return {"TFLOPs": flops * n / dt / 1e12, "frac_of_mfma_peak": flops * n / dt / 1e12 / PEAK_MFMA_F16_TFLOPS, "launches": n, "seconds": dt,
            "what": "register-only loop of v_mfma_f32_32x32x16_f16 on N(0,1) x N(0,0.02) operands, 256 workgroups of 8 waves, "
                    "back-to-back launches of about 4 ms: the rate the board's power management grants the MFMA unit "
                    "with no data movement at all"}


def run_small_batch_sweep(args):
    """The setting of the paper's ablation on hiding the recomputation (Sec. 4.5, Table 2): OPT-6.7B shape, prompt 256,
    small batches, weights offloaded, one GPU batch, so that a layer's weights (384 MiB) arrive long after its cache.
    Three arms per batch size: no recomputation (l = 0), the planned split with the recomputation waiting for the whole
    layer's weights, and with the fine-grained pipeline ([Wk;Wv] first)."""
    say = lambda msg: print("bench: " + msg, file=sys.stderr, flush=True)
    rows = []
    layers = 8 if args.layers == 40 else args.layers      # 8 layers (3 GiB of pinned weights) unless --layers says otherwise
    for b in (1, 2, 4, 8, 16, 32):
        say(f"small-batch sweep: batch {b}")
        a = argparse.Namespace(**vars(args))
        a.model, a.batch, a.seq, a.layers, a.gpu_batches, a.gen, a.warmup = "opt-6.7b", b, 256, layers, 1, args.gen, 2
        a.weight_pipeline_ablation, a.extension_chunks = True, 0
        r = run_columns(a)
        rows.append({"batch": b, "kv_cache_MiB_per_layer": 2 * b * 256 * 4096 * 2 / 2**20, "split": r["kvpr"]["split"],
                     "tokens_per_s": {"no_recompute": r["no_recompute"]["tokens_per_s"],
                                      "kvpr_without_weight_pipeline": r["kvpr_without_weight_pipeline"]["tokens_per_s"],
                                      "kvpr": r["kvpr"]["tokens_per_s"]}})
    print(json.dumps({"what": "decode tokens/s, OPT-6.7B-shaped layers with offloaded weights, context 256, one GPU batch (the setting of the "
                              "paper's Table 2)", "layers": layers, "tokens": args.gen, "rows": rows}))


def token_gemm_rooflines(model, b, launches=30):
    """The four weight-streaming GEMMs of a decoder layer for the decode token (q|k|v, output projection, FFN up, FFN
    down) at `model`'s width, launched as a context launches them (with its K-slice workspace), back to back over
    rotating copies of the weights (more than the 256 MiB memory-side cache holds) between one pair of events.
    Algorithmic bytes = the weight matrix once."""
    import torch
    import kvpr_inputs
    import paper_2411_17089_amd as k
    h = kvpr_inputs.SHAPES[model][0]
    g = torch.Generator(device="cuda").manual_seed(1)
    ws_bytes = k.kvpr_token_gemm_workspace_bytes(b, h)
    ws = torch.zeros(ws_bytes, dtype=torch.uint8, device="cuda")
    out = []
    for name, N, K in (("q|k|v", 3 * h, h), ("output projection", h, h), ("FFN up", 4 * h, h), ("FFN down", h, 4 * h)):
        x = torch.randn((b, K), device="cuda", dtype=torch.float32, generator=g).half()
        copies = max(2, int(600e6 // (N * K * 2)) + 1)
        Ws = [(torch.randn((N, K), device="cuda", dtype=torch.float32, generator=g) * 0.02).half() for _ in range(copies)]
        y = torch.empty((b, N), device="cuda", dtype=torch.float16)
        def launch(i):
            k.kvpr_token_gemm_ws(x, Ws[i % copies], None, None, y, b, N, K, 0, N, ws, ws_bytes)
        for i in range(5):
            launch(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(launches):
            launch(i)
        e1.record()
        e1.synchronize()
        us = e0.elapsed_time(e1) / launches * 1e3
        byt = N * K * 2
        out.append({"gemm": name, "M": b, "N": N, "K": K, "bytes": byt, "avg_us": us, "achieved_GBps": byt / us / 1e3,
                    "frac_of_hbm_peak": byt / us / 1e3 / PEAK_HBM_GBPS})
        del Ws
    return {"bound": "hbm", "peak": PEAK_HBM_GBPS, "unit": "GB/s", "launches_back_to_back": launches, "shape": model, "gemms": out}


def headline(args, r):
    """The one-line record of the driver's contract, from the figures of one layer case."""
    pf = profile_figures(r["model"], r["batch"], r["context"])
    traffic = None
    roof = {"kernel": "gemm_bias_f16 (recompute GEMM%s)" % (", rotary epilogue" if r["model"].startswith("llama") else ""),
            "bound": "mfma", "achieved": r["gemm"]["TFLOPs"], "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s",
            "frac": r["gemm"]["frac_of_mfma_peak"], "traffic": None, "flops_per_launch": r["gemm"]["flops_per_launch"],
            "avg_ms": r["gemm"]["avg_ms"],
            "measured": "HIP events around the launch inside each timed layer decode, mean over the timed steps"}
    if pf:
        # not measurable inside this process: counters of a separate rocprofv3 run of `bench.py --kernels` at this shape,
        # per recomputed position (the kernel's traffic is linear in the number of row tiles), times this run's split
        traffic = (pf["fetch_bytes_per_position"] + pf["write_bytes_per_position"]) * r["split"]
        roof["traffic"] = traffic
        roof["traffic_source"] = pf.get("source", "profiles/traffic.json")
        roof["traffic_detail"] = {"fetch_bytes": pf["fetch_bytes_per_position"] * r["split"],
                                  "write_bytes": pf["write_bytes_per_position"] * r["split"],
                                  "algorithmic_read_bytes": 2.0 * r["batch"] * r["split"] * pf["hidden"] + 4.0 * pf["hidden"] ** 2,
                                  "algorithmic_write_bytes": 4.0 * r["batch"] * r["split"] * pf["hidden"]}
        if "mfma_busy_frac" in pf:
            roof["mfma_busy_frac"] = pf["mfma_busy_frac"]
            roof["mfma_busy_source"] = pf.get("mfma_busy_source", roof["traffic_source"])
    out = {
        "metric": "decode_layer_tokens_per_s_at_optimal_split",
        "value": r["tokens_per_s"],
        "unit": "tokens/s per layer (batch / per-layer decode latency)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": r["ms_per_layer"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic (seeded N(0,1) activations, N(0,0.02) weights; cache = GPU prefill of the same X)",
        "config": {"workload": r["workload"], "cost_model": args.cost_model, "granularity": args.granularity,
                   "l_star": r["l_star"], "chunks": args.chunks, "store_int4": args.store_int4},
        "ms_per_layer": r["ms_per_layer"], "ms_assemble": r["ms_assemble"], "ms_total_events": r["ms_total_events"],
        "ms_total_events_min_median_max": r["ms_total_events_min_median_max"],
        "bounds": r["bounds"],
        "latency_over_bound": r["bounds"]["assemble_over_plain_eq10_at_split"],
        "breakdown_ms": r["breakdown_ms"], "profile": r["profile"],
        "roofline": roof,
        "h2d": r["h2d"],
    }
    if "attention" in r:
        a = r["attention"]["as_in_layer"]
        out["roofline_attention"] = {"kernel": a["kernels"] + ", float16 cache, as the layer launches it at this split, 20 times back to back",
                                     "bound": "hbm", "achieved": a["GBps"], "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                     "frac": a["frac_of_hbm_peak"], "bytes_per_launch": r["attention"]["bytes_per_launch"],
                                     "avg_ms": a["avg_ms"], "single_launch": r["attention"]["single_launch"],
                                     "in_layer_event_pairs": r["attention_in_layer_event_pairs"]}
    for key in ("extension_chunked_copy", "split_sweep", "cpu_baseline", "without_keep_warm", "keep_warm_fraction"):
        if key in r:
            out[key] = r[key]
    return out


def compact(r):
    """A case as an entry of the `configs` array."""
    e = {"workload": r["workload"], "l_star": r["l_star"], "l_star_from_startup_profile_alone": r["l_star_from_startup_profile_alone"],
         "ms_per_layer": r["ms_per_layer"], "tokens_per_s": r["tokens_per_s"],
         "gemm_TFLOPs": r["gemm"]["TFLOPs"], "gemm_frac_of_mfma_peak": r["gemm"]["frac_of_mfma_peak"],
         "gemm_median_TFLOPs": r["gemm"]["median_TFLOPs"],
         "h2d_GBps": r["h2d"]["achieved_GBps"], "h2d_frac_of_pinned_peak": r["h2d"]["frac"], "h2d_median_GBps": r["h2d"]["median_GBps"],
         "assemble_over_builder_bound": r["bounds"]["assemble_over_builder_bound"],
         "assemble_over_plain_eq10_at_split": r["bounds"]["assemble_over_plain_eq10_at_split"],
         "assemble_over_plain_eq10_optimum": r["bounds"]["assemble_over_plain_eq10_optimum"],
         "plain_eq10_l_star": r["bounds"]["plain_eq10_l_star"], "ms_total_events_min_median_max": r["ms_total_events_min_median_max"],
         "profile": {"v_com_GBps": r["profile"]["v_com_GBps"], "v_gpu_TFLOPs": r["profile"]["v_gpu_TFLOPs"],
                     "before_calibration": r["profile"]["before_calibration"],
                     "calibration_link_ms_gemm_ms": r["profile"]["calibration_link_ms_gemm_ms"]}}
    if "attention" in r:
        e["attention_frac_of_hbm_peak_as_in_layer"] = r["attention"]["as_in_layer"]["frac_of_hbm_peak"]
        e["attention_frac_of_hbm_peak_single_launch"] = r["attention"]["single_launch"]["frac_of_hbm_peak"]
    for key in ("split_sweep", "extension_chunked_copy", "without_keep_warm"):
        if key in r:
            e[key] = r[key]
    return e


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed decodes before the timed ones, enqueued like them: the first burst of a given size makes the runtime grow its "
                         "pools, and work running meanwhile takes up to twice as long.  Default max(25, steps); 2 tokens in --stack / --columns mode")
    ap.add_argument("--model", default=None,
                    help="opt-6.7b | opt-13b | opt-30b | llama2-7b | llama2-13b | tiny: run this one layer shape; default = every configuration")
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--seq", type=int, default=1024)
    ap.add_argument("--split", type=int, default=-1, help="-1 = scheduler's l*")
    ap.add_argument("--cost-model", default="eq10", choices=["eq10", "ns", "row", "pipe"])
    ap.add_argument("--stack", action="store_true", help="layer-pipelined decode of a whole stack instead of one layer")
    ap.add_argument("--columns", action="store_true",
                    help="throughput mode: column-by-column schedule with the weights offloaded too (use with --layers, --gpu-batches)")
    ap.add_argument("--gpu-batches", type=int, default=4)
    ap.add_argument("--small-batch-sweep", action="store_true", help="column schedule at batch 1..32, context 256, OPT-6.7B shape: no recomputation / planned split without / with the fine-grained weight pipeline (the setting of the paper's Table 2); --layers and --gen apply")
    ap.add_argument("--weight-pipeline-ablation", action="store_true", help="--columns: also time the planned split with the recomputation waiting for the whole layer's weights")
    ap.add_argument("--hidden-offload", action="store_true", help="--columns: keep the hidden states between layers in pinned host memory (Algorithm 1)")
    ap.add_argument("--kernels", action="store_true", help="launch each kernel of the path standalone (for rocprofv3 --pmc runs)")
    ap.add_argument("--power-probe", action="store_true",
                    help="clock / power evidence: the recompute GEMM and a register-only MFMA loop on normal, constant and zero operands under amd-smi sampling")
    ap.add_argument("--probe-seconds", type=float, default=6.0)
    ap.add_argument("--layers", type=int, default=40)
    ap.add_argument("--gen", type=int, default=32)
    ap.add_argument("--no-greedy", action="store_true", help="(stack mode, diagnostics) skip the LM head / argmax / embedding step")
    ap.add_argument("--granularity", type=int, default=64,
                    help="l is restricted to multiples of this: 64 positions x batch 32 = 8 GEMM tile rows = a whole number of 256-workgroup rounds at hidden 4096")
    ap.add_argument("--chunks", type=int, default=1,
                    help="extension: copy X[0:l] in this many parts and start each part's GEMM as it lands (1 = paper's schedule)")
    ap.add_argument("--extension-chunks", type=int, default=3,
                    help="after the timed region, also measure the chunked-copy extension with this many parts (0 = skip)")
    ap.add_argument("--store-int4", default="none", choices=["none", "kv", "both"],
                    help="keep the host store group-wise 4-bit compressed (Sec. 4.4): the cache only, or the cache and the activations")
    ap.add_argument("--adaptive", type=float, default=0.0,
                    help="(stack / columns modes) extension: keep adapting v_com / v_gpu while decoding with this moving-average weight")
    ap.add_argument("--calibrate", type=int, default=6,
                    help="untimed decodes whose median link and GEMM rates replace the profiled v_com / v_gpu before planning (0 = plan from the profiler alone)")
    ap.add_argument("--keep-warm", type=float, default=0.85,
                    help="extension: fraction of the predicted activation-copy time during which the otherwise idle GPU runs a "
                         "register-only MFMA loop, so that the recompute GEMM does not start with the clocks down (0 = off)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seqs", type=int, default=32)
    ap.add_argument("--skip", default="", help="comma list of parts to leave out: ceiling, token_gemm; in the default run also sweep, stack, columns")
    args = ap.parse_args()
    if args.warmup is None:
        args.warmup = 2 if (args.stack or args.columns) else max(25, args.steps)
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2411_17089_amd as k  # noqa: F401  (fails loudly when libkvpr.so is missing)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    say = lambda msg: print("bench: " + msg, file=sys.stderr, flush=True)
    if args.stack:
        args.model = args.model or "opt-13b"
        return print(json.dumps(run_stack(args)))
    if args.kernels:
        args.model = args.model or "opt-6.7b"
        return run_kernels(args)
    if args.power_probe:
        args.model = args.model or "opt-6.7b"
        return run_power_probe(args)
    if args.small_batch_sweep:
        return run_small_batch_sweep(args)
    if args.columns:
        args.model = args.model or "opt-13b"
        return print(json.dumps(run_columns(args)))
    if args.model is not None:
        r = run_layer(args, args.model, args.batch, args.seq, args.split, attention=True, extension=True,
                      cpu=not args.no_cpu_baseline)
        result = headline(args, r)
        if "token_gemm" not in args.skip.split(","):
            result["roofline_token_gemm"] = token_gemm_rooflines(args.model, args.batch)
        if "ceiling" not in args.skip.split(","):
            ceil = mfma_ceiling()
            result["roofline"]["power_limited_mfma_ceiling"] = ceil
            result["roofline"]["achieved_over_power_limited_ceiling"] = result["roofline"]["achieved"] / ceil["TFLOPs"]
        return print(json.dumps(result))

    # ---- default: every configuration the metric is quoted on, one JSON line ----
    skip = set(filter(None, args.skip.split(",")))
    t_start = time.perf_counter()
    configs = []
    say("OPT-6.7B shape, batch 32, context 1024 (l* and the split sweep, CPU oracle beside it)")
    c2 = run_layer(args, "opt-6.7b", 32, 1024, sweep=() if "sweep" in skip else (0, 256, 512, 768, 1024), extension=True,
                   cpu=not args.no_cpu_baseline)
    say("OPT-13B shape, batch 32, context 1024")
    c3 = run_layer(args, "opt-13b", 32, 1024)
    say("OPT-30B shape, batch 32, context 1024 (headline)")
    c4 = run_layer(args, "opt-30b", 32, 1024, extension=True)
    configs += [compact(c2), compact(c3)]
    if "sweep" not in skip:
        for s in (512, 1024, 2048, 4096):
            say(f"OPT-30B shape, batch 16, context {s}")
            configs.append(compact(run_layer(args, "opt-30b", 16, s)))
    result = headline(args, c4)
    if "token_gemm" not in skip:
        say("token GEMMs of a decoder layer at the headline width")
        result["roofline_token_gemm"] = token_gemm_rooflines("opt-30b", 32)
    if "ceiling" not in skip:
        say("register-only MFMA loop (what the power limit grants on this data)")
        ceil = mfma_ceiling()
        result["roofline"]["power_limited_mfma_ceiling"] = ceil
        result["roofline"]["achieved_over_power_limited_ceiling"] = result["roofline"]["achieved"] / ceil["TFLOPs"]
    if "cpu_baseline" in c2:
        result["cpu_baseline"] = c2["cpu_baseline"]
        result["cpu_baseline"]["note"] = ("timed on the OPT-6.7B-shaped layer (first entry of configs), not on the headline shape: the "
                                          "float64 oracle needs (7168/4096)^2 = 3.1 times as long per sequence there")
    if "stack" not in skip:
        say("OPT-13B-shaped stack, 40 layers, batch 32, prompt 1024, 32 greedy tokens")
        sa = argparse.Namespace(**vars(args))
        sa.model, sa.batch, sa.seq, sa.layers, sa.gen, sa.warmup = "opt-13b", 32, 1024, 40, 32, 2
        st = run_stack(sa)
        configs.append({"workload": st["config"]["workload"], "tokens_per_s": st["value"], "ms_per_token": st["ms_per_step"],
                        "ms_per_layer": st["ms_per_layer"], "splits_first_last": st["config"]["splits_first_last"],
                        "h2d_GBps_sustained": st["h2d_GBps_sustained"], "h2d_frac_of_peak": st["h2d_frac_of_peak"],
                        "breakdown_ms_per_layer": st["breakdown_ms_per_layer"], "host_enqueue_ms_per_token": st["host_enqueue_ms_per_token"],
                        "pinned_store_GiB": st["pinned_store_GiB"], "profile": st["profile"], "cost_model": st["config"]["cost_model"]})
        if "extension_steady_state_cost_form" in st:
            configs[-1]["extension_steady_state_cost_form"] = st["extension_steady_state_cost_form"]
    if "columns" not in skip:
        say("column-by-column schedule, OPT-13B shape, 8 layers x 4 GPU batches of 32, weights offloaded")
        ca = argparse.Namespace(**vars(args))
        ca.model, ca.batch, ca.seq, ca.layers, ca.gpu_batches, ca.gen, ca.warmup = "opt-13b", 32, 1024, 8, 4, 8, 2
        co = run_columns(ca)
        configs.append({"workload": co["config"]["workload"], "tokens_per_s": co["value"], "kvpr": co["kvpr"],
                        "no_recompute": co["no_recompute"], "speedup_over_no_recompute": co["speedup_over_no_recompute"]})
        if "extension_steady_state_cost_form" in co:
            configs[-1]["extension_steady_state_cost_form"] = co["extension_steady_state_cost_form"]
    result["configs"] = configs
    result["bench_wall_s"] = time.perf_counter() - t_start
    print(json.dumps(result))


if __name__ == "__main__":
    main()
