#!/usr/bin/env python3
"""Bench of KVPR's per-layer decode hot path on one MI355X.

A "step" is one decode of one OPT-6.7B-shaped attention layer (hidden 4096, 32 heads x 128,
fp16, batch 32, context 1024) through the whole path at the scheduler-chosen split l*:
H2D of X[0:l*] and KV[l*:s] from the pinned host store, new-token q/k/v projection, recompute
GEMM, decode attention over s+1 positions, output projection, store-back.  The layer's
activations and cache start in pinned host memory (that is where the method keeps them; moving
them is the method), weights and the decode token's input are resident in HBM.

Prints ONE JSON line.  Paper context (A100 + PCIe 4.0, whole models, not comparable): up to
35.8 % lower decode latency and 46.2 % higher throughput than its baselines.
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
    ctx = k.kvpr_create(L, h, H, d, ffn, b, s + gen + args.warmup + 2, dtype=k.KVPR_F16 | qflags,
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
        "pinned_store_GiB": L * (s + gen + args.warmup + 2) * (x_bpp + kv_bpp) / 2 ** 30, "setup_s": setup_s,
    }
    k.kvpr_destroy(ctx)
    print(json.dumps(result))


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
    ctx = k.kvpr_create_offload(L, h, H, d, ffn, b, s + 2 * (gen + args.warmup) + 2, nb, dtype=k.KVPR_F16 | qflags,
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
    x = (torch.randn((nb, b, h), device="cuda") * 1.0).half()
    x_out = torch.empty_like(x)
    seq = s
    results = {}
    for name, splits in (("kvpr", None), ("no_recompute", [0] * S)):
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
        "speedup_over_no_recompute": results["no_recompute"]["ms_per_token_step"] / r["ms_per_token_step"],
        "profile": {"v_com_GBps": prof.h2d_bytes_per_s / 1e9, "v_gpu_TFLOPs": prof.gemm_flops_per_s / 1e12},
        "pinned_GiB": (S * (s + 2 * (gen + args.warmup) + 2) * (x_bpp + kv_bpp) + L * blob_bytes) / 2 ** 30, "setup_s": setup_s,
    }
    k.kvpr_destroy(ctx)
    print(json.dumps(out))


def run_kernels(args):
    """Standalone launches of the path's kernels at the bench shape, for rocprofv3 counter runs:
    a plain device copy of known size (reference for scaling FETCH_SIZE / WRITE_SIZE), the recompute
    GEMM at M = split*batch, decode attention over seq+1 positions, and the two token GEMMs."""
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
    timed("token_gemm_qkv_ms", lambda: k.kvpr_token_gemm(x, W, bias, q, y16, b, 3 * h, h, h, 2 * h))
    timed("token_gemm_out_ms", lambda: k.kvpr_token_gemm(x, W, bias, None, y16, b, h, h, 0, h))
    out["recompute_gemm_TFLOPs"] = 4.0 * M * h * h / out["recompute_gemm_ms"] / 1e9
    out["attention_GBps"] = 2.0 * b * (s + 1) * h * 2 / out["attention_ms"] / 1e6
    out["shape"] = {"model": args.model, "batch": b, "seq": s, "split": split, "M": M, "N": 2 * h, "K": h}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--model", default="opt-6.7b", help="opt-6.7b | opt-13b | opt-30b | llama2-7b | llama2-13b | tiny")
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--seq", type=int, default=1024)
    ap.add_argument("--split", type=int, default=-1, help="-1 = scheduler's l*")
    ap.add_argument("--cost-model", default="eq10", choices=["eq10", "ns", "row", "pipe"])
    ap.add_argument("--stack", action="store_true", help="layer-pipelined decode of a whole stack instead of one layer")
    ap.add_argument("--columns", action="store_true",
                    help="throughput mode: column-by-column schedule with the weights offloaded too (use with --layers, --gpu-batches)")
    ap.add_argument("--gpu-batches", type=int, default=4)
    ap.add_argument("--kernels", action="store_true", help="launch each kernel of the path standalone (for rocprofv3 --pmc runs)")
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
                    help="untimed decodes that refine the profiled v_com / v_gpu inside the real pipeline before planning (0 = plan from kvpr_profile alone)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seqs", type=int, default=32)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import kvpr_inputs
    import paper_2411_17089_amd as k

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.stack:
        return run_stack(args)
    if args.kernels:
        return run_kernels(args)
    if args.columns:
        return run_columns(args)
    h, H, d = kvpr_inputs.SHAPES[args.model]
    b, s = args.batch, args.seq
    cm = {"eq10": k.KVPR_COST_EQ10, "ns": k.KVPR_COST_NS, "row": k.KVPR_COST_ROW, "pipe": k.KVPR_COST_PIPE}[args.cost_model]

    layer = kvpr_inputs.make_layer(0, b, s, h, H)
    f16 = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    llama = args.model.startswith("llama")
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

    prof0 = k.kvpr_profile(ctx, b, s)
    k.kvpr_set_profile(ctx, prof0, cm, args.granularity)
    k.kvpr_set_chunks(ctx, args.chunks)
    # Refine the two constants in place: a few untimed decodes at the planned split with the run-time adaptation on.
    # The GEMM inside the real pipeline (fresh activations, cache copy in flight, GPU coming out of an idle stretch)
    # runs up to 15 % below its isolated rate on the wider shapes; the plan should use what the pipeline delivers.
    prof = prof0
    if args.calibrate > 0 and args.split < 0:
        k.kvpr_set_adaptive(ctx, 0.5)
        for _ in range(args.calibrate):
            k.kvpr_layer_decode(ctx, 0, s, -1, w, x_new, out)
            torch.cuda.synchronize()
        prof = k.kvpr_get_profile(ctx)
        k.kvpr_set_adaptive(ctx, 0.0)
    pchunks = args.chunks if cm == k.KVPR_COST_EQ10 else 1
    # the split comes from the calibrated constants; every "bound" below is the cost model with the start-up profile's
    # constants (isolated copy rate, GEMM under a concurrent copy), so that the ratios are not measured against themselves
    l_star, t_bound = k.kvpr_plan_split_linear(prof, cm, pchunks, s, x_bpp, kv_bpp, f_pp, args.granularity)
    split = l_star if args.split < 0 else args.split
    t_bound_split = k.kvpr_cost_linear(prof0, cm, pchunks, split, s, x_bpp, kv_bpp, f_pp)
    l_eq10, t_eq10 = k.kvpr_plan_split_linear(prof0, k.KVPR_COST_EQ10, 1, s, x_bpp, kv_bpp, f_pp, args.granularity)

    for _ in range(args.warmup):
        k.kvpr_layer_decode(ctx, 0, s, split, w, x_new, out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        k.kvpr_layer_decode_timed(ctx, 0, s, split, w, x_new, out, i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    tim = [k.kvpr_timing_read(ctx, i) for i in range(args.steps)]
    ms_step = wall * 1e3 / args.steps

    mean = lambda name: float(np.mean([getattr(t, name) for t in tim]))
    ms_gemm, ms_attn = mean("ms_recompute"), mean("ms_attn")
    ms_act, ms_kv = mean("ms_act_copy"), mean("ms_kv_copy")
    gemm_flops = 4.0 * b * split * h * h
    attn_bytes = 2.0 * b * (s + 1) * h * 2
    # ms_attn sums the two attention phases; with a packed cache the transferred rows are read in packed form
    attn_phase_bytes = float(2 * b * (split + 1) * h * 2 + kv_bpp * (s - split)) if qflags & k.KVPR_KV_INT4 else attn_bytes
    attn_kernel = ("attention_partial_ranged x2 (+combine)" if (qflags & k.KVPR_KV_INT4 or split >= 128)
                   else "attention_partial (+combine)")
    h2d_bytes = float(x_bpp * split + kv_bpp * (s - split))
    gemm_tflops = gemm_flops / (ms_gemm * 1e-3) / 1e12 if split > 0 else 0.0
    attn_gbps = attn_phase_bytes / (ms_attn * 1e-3) / 1e9
    h2d_gbps = h2d_bytes / ((ms_act + ms_kv) * 1e-3) / 1e9

    # the attention kernel again, 20 launches back to back between one pair of events on the same stream: the
    # per-layer event pair above also holds the two event-to-kernel gaps (~10 us of a ~90 us kernel)
    kv_res = torch.randn((s + 1, b, 2 * h), dtype=torch.float16, device="cuda")
    q_res = torch.randn((b, h), dtype=torch.float32, device="cuda")
    z_res = torch.empty((b, h), dtype=torch.float16, device="cuda")
    ws_res = torch.empty(k.kvpr_attention_workspace_bytes(b, h, H, s + 1), dtype=torch.uint8, device="cuda")
    for _ in range(3):
        k.kvpr_decode_attention(q_res, kv_res, z_res, ws_res, s + 1, b, h, H)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        k.kvpr_decode_attention(q_res, kv_res, z_res, ws_res, s + 1, b, h, H)
    e1.record()
    e1.synchronize()
    ms_attn_b2b = e0.elapsed_time(e1) / 20
    del kv_res
    attn_gbps_b2b = attn_bytes / (ms_attn_b2b * 1e-3) / 1e9

    # HBM-side bytes per launch from the committed rocprofv3 --pmc runs (FETCH_SIZE + WRITE_SIZE, scaled by a
    # known-size copy); only valid for the shape and split they were taken at
    traffic, traffic_detail = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        traffic_detail = json.load(open(tpath)).get(f"recompute_gemm/{args.model}/b{b}/s{s}")
        if traffic_detail and traffic_detail.get("split") == split:
            traffic = traffic_detail["total_bytes"]
        else:
            traffic_detail = None

    result = {
        "metric": "decode_layer_tokens_per_s_at_optimal_split",
        "value": b / (ms_step * 1e-3),
        "unit": "tokens/s per layer (batch / per-layer decode latency)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic (seeded N(0,1) activations, N(0,0.02) weights; cache = GPU prefill of the same X)",
        "config": {"workload": f"{args.model}-shaped attention layer, hidden {h}, {H} heads x {d}, batch {b}, context {s}, "
                               f"decode 1 token at split l={split}",
                   "cost_model": args.cost_model, "granularity": args.granularity, "l_star": l_star, "chunks": args.chunks,
                   "store_int4": args.store_int4},
        "ms_per_layer": ms_step,
        "ms_assemble": mean("ms_assemble"), "ms_total_events": mean("ms_total"),
        # per-step spread (event time first enqueue -> end of the step): the link of these boxes has occasional slow stretches
        "ms_total_events_min_median_max": [float(np.min([t.ms_total for t in tim])), float(np.median([t.ms_total for t in tim])),
                                           float(np.max([t.ms_total for t in tim]))],
        "cost_model_bound_ms": t_bound_split * 1e3,
        "eq10_bound_ms_at_its_own_optimum": t_eq10 * 1e3, "eq10_l_star": l_eq10,
        "step_over_eq10_bound": ms_step / (t_eq10 * 1e3),
        "latency_over_bound": mean("ms_assemble") / (t_bound_split * 1e3),
        "step_over_bound": ms_step / (t_bound_split * 1e3),
        "breakdown_ms": {"act_copy": ms_act, "kv_copy": ms_kv, "recompute": ms_gemm, "proj": mean("ms_proj"),
                         "attn": ms_attn, "out": mean("ms_out"), "store": mean("ms_store"), "attn_early": mean("ms_attn_early")},
        "profile": {"v_com_GBps": prof.h2d_bytes_per_s / 1e9, "v_gpu_TFLOPs": prof.gemm_flops_per_s / 1e12,
                    "before_calibration": {"v_com_GBps": prof0.h2d_bytes_per_s / 1e9, "v_gpu_TFLOPs": prof0.gemm_flops_per_s / 1e12},
                    "calibration_decodes": args.calibrate if args.split < 0 else 0,
                    "v_gpu_alone_TFLOPs": prof.gemm_alone_flops_per_s / 1e12, "h2d_peak_GBps": prof.h2d_peak_bytes_per_s / 1e9, "d2h_GBps": prof.d2h_bytes_per_s / 1e9,
                    "attn_GBps": prof.attn_bytes_per_s / 1e9},
        "roofline": {"kernel": "gemm_bias_f16 (recompute GEMM%s)" % (", rotary epilogue" if llama else ""), "bound": "mfma", "achieved": gemm_tflops,
                     "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s", "frac": gemm_tflops / PEAK_MFMA_F16_TFLOPS,
                     "traffic": traffic, "traffic_detail": traffic_detail, "flops_per_launch": gemm_flops, "avg_ms": ms_gemm},
        # the attention kernel by itself: one pass over all s+1 float16 rows, 20 launches between one pair of events
        # (the in-layer figures below are event pairs around single ~30-90 us launches and carry ~10 us of gap each)
        "roofline_attention": {"kernel": "attention_partial (+combine), float16 cache, back to back", "bound": "hbm",
                               "achieved": attn_gbps_b2b, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                               "frac": attn_gbps_b2b / PEAK_HBM_GBPS, "bytes_per_launch": attn_bytes, "avg_ms": ms_attn_b2b,
                               "in_layer": {"kernels": attn_kernel, "ms": ms_attn, "ms_before_cache_fence": mean("ms_attn_early"),
                                            "bytes": attn_phase_bytes, "GBps": attn_gbps}},
        "h2d": {"achieved_GBps": h2d_gbps, "measured_pinned_peak_GBps": prof.h2d_peak_bytes_per_s / 1e9,
                "frac": h2d_gbps / (prof.h2d_peak_bytes_per_s / 1e9), "bytes_per_step": h2d_bytes},
    }

    if args.extension_chunks > 1 and args.chunks == 1 and cm == k.KVPR_COST_EQ10 and args.split < 0:
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
        result["extension_chunked_copy"] = {
            "chunks": c, "l_star": l_c, "ms_per_layer": ms_c, "tokens_per_s": b / (ms_c * 1e-3),
            "chunked_model_bound_ms": t_c * 1e3, "step_over_chunked_bound": ms_c / (t_c * 1e3),
            "step_over_eq10_bound": ms_c / (t_eq10 * 1e3), "speedup_over_paper_schedule": ms_step / ms_c,
            "note": "not the paper's schedule: X[0:l] travels in parts and each part is recomputed as it lands; "
                    "same outputs bit for bit"}

    if not args.no_cpu_baseline:
        n_seq = min(args.cpu_seqs, b)
        o_ref, dt, cores = cpu_baseline(layer, n_seq, llama)
        got = out.float().cpu().numpy()[:n_seq]
        result["cpu_baseline"] = {
            "value": n_seq / dt, "unit": "tokens/s per layer", "cores": cores, "kind": "oracle",
            "sample": f"first {n_seq} of the {b} sequences of the same layer, one decode step: numpy float64 recompute of "
                      f"all {s} K/V rows (Eq. 1) + attention + output projection; {dt:.2f} s",
            ("max_rel_err_gpu_vs_oracle_on_sample" if not qflags else "max_rel_err_gpu_over_4bit_store_vs_exact_oracle_on_sample"):
                float(np.max(np.abs(got - o_ref)) / np.max(np.abs(o_ref))),
        }
    k.kvpr_destroy(ctx)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
