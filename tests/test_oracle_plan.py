"""Pins for oracle/kvpr_plan_oracle.py: the paper's Table 1, its split-point figure,
closed forms of the piecewise-linear cost, limits and a hand-evaluated toy."""
import json
import math
import os

import pytest

from oracle import kvpr_plan_oracle as po


# ---- P8: size closed forms (Eq. 6, Eq. 8) against Table 1 --------------------
def test_table1_kv_sizes_and_pcie_time(golden_dir):
    t1 = json.load(open(os.path.join(golden_dir, "table1_kv_sizes.json")))
    b, s, p = t1["batch"], t1["seq"], t1["elem_bytes"]
    for row in t1["rows"]:
        h = row["hidden"]
        kv = po.bytes_kv(b, 0, s, h, p)
        assert kv == row["kv_MB"] * 2 ** 20
        assert po.bytes_x(b, s, h, p) * 2 == kv
        # the printed PCIe latency is size / 32 GiB/s, to the printed 3 digits
        t0 = po.cost(po.COST_EQ10, 0, b, s, h, p, 32 * 2.0 ** 30, 1e15)
        assert abs(t0 * 1e3 - row["pcie_ms"]) < 0.05
        assert po.cost(po.COST_ROW, 0, b, s, h, p, 32 * 2.0 ** 30, 1e15) == t0


def test_recompute_flops_are_two_gemms():
    # K and V projections of b*l rows: 2 GEMMs of [b*l, h] x [h, h], 2 flops per multiply-add
    for b, l, h in [(32, 1024, 4096), (1, 7, 768), (16, 4096, 7168)]:
        assert po.flops_recompute(b, l, h) == 2 * (2 * (b * l) * h * h)
    assert po.flops_recompute(32, 1024, 4096) == 2199023255552
    assert po.flops_recompute(32, 1024, 5120) == 3435973836800
    assert po.flops_recompute(32, 1024, 7168) == 6734508720128


# ---- P7: hand-evaluated toy ----------------------------------------------------
def _toy():
    # per position: activation copy 1 s, KV copy 2 s, recompute 1 s  (b=h=1... use b*h*p = 1 byte units)
    # b=1,h=1,p=1: M_X = l, M_KV = 2(s-l), N = 4l ; v_com = 1 B/s, v_gpu = 4 flop/s
    return dict(b=1, s=9, h=1, p=1, v_com=1.0, v_gpu=4.0)


def test_toy_cost_curves():
    k = _toy()
    e10 = [po.cost(po.COST_EQ10, l, **k) for l in range(10)]
    ns = [po.cost(po.COST_NS, l, **k) for l in range(10)]
    row = [po.cost(po.COST_ROW, l, **k) for l in range(10)]
    # by hand: t_act=l, t_kv=2(9-l), t_rc=l
    assert e10 == [18, 17, 16, 15, 14, 13, 12, 14, 16, 18]
    assert ns == [18, 16, 14, 12, 10, 10, 12, 14, 16, 18]
    assert row == [18, 16, 14, 12, 10, 8, 6, 7, 8, 9]
    assert po.plan_split(po.COST_EQ10, **k) == (6, 12.0)
    assert po.plan_split(po.COST_NS, **k) == (4, 10.0)        # tie 4/5 -> smallest
    assert po.plan_split(po.COST_ROW, **k) == (6, 6.0)


def test_pipelined_extension_toy():
    # link = l + 2(9-l) = 18 - l, recompute = l: max crosses at l = 9
    k = _toy()
    assert [po.cost(po.COST_PIPE, l, **k) for l in range(10)] == [18, 17, 16, 15, 14, 13, 12, 11, 10, 9]
    assert po.plan_split(po.COST_PIPE, **k) == (9, 9.0)
    k["v_gpu"] = 1.0                                   # recompute 4 s per position: 18 - l meets 4l at l = 3.6
    assert [po.cost(po.COST_PIPE, l, **k) for l in (3, 4)] == [15, 16]
    assert po.plan_split(po.COST_PIPE, **k) == (3, 15.0)


def test_limits():
    kw = dict(b=32, s=1024, h=4096, p=2, v_com=50e9)
    assert po.plan_split(po.COST_EQ10, v_gpu=1e30, **kw)[0] == 1024     # free compute: recompute everything
    assert po.plan_split(po.COST_ROW, v_gpu=1e30, **kw)[0] == 1024
    assert po.plan_split(po.COST_EQ10, v_gpu=1e3, **kw)[0] == 0         # no compute: transfer everything
    l, t = po.plan_split(po.COST_EQ10, v_gpu=1e3, **kw)
    assert t == po.bytes_kv(32, 0, 1024, 4096, 2) / 50e9


# ---- P6: closed form of the real-valued optimum ---------------------------------
def _lx(model, s, h, p, v_com, v_gpu):
    rho = 2.0 * h * v_com / (p * v_gpu)
    return s / ((1.5 if model == po.COST_NS else 1.0) + rho)


@pytest.mark.parametrize("model", [po.COST_EQ10, po.COST_ROW, po.COST_NS])
@pytest.mark.parametrize("b,s,h,v_com,v_gpu", [
    (32, 1024, 4096, 57e9, 1.2e15), (1, 128, 768, 20e9, 3e13), (16, 4096, 7168, 55e9, 9e14),
    (4, 37, 64, 1e9, 5e11), (2, 1000, 5120, 32e9, 312e12)])
def test_argmin_brackets_closed_form(model, b, s, h, v_com, v_gpu):
    l, t = po.plan_split(model, b, s, h, 2, v_com, v_gpu)
    lx = _lx(model, s, h, 2, v_com, v_gpu)
    assert l in (math.floor(lx), math.ceil(lx))
    # brute-force property: nothing beats it, and it is the first minimum
    ts = [po.cost(model, k, b, s, h, 2, v_com, v_gpu) for k in range(s + 1)]
    assert t == min(ts) and l == ts.index(min(ts))
    # proportionality: l*/s' is (nearly) constant as the sequence grows
    l2, _ = po.plan_split(model, b, 2 * s, h, 2, v_com, v_gpu)
    assert abs(l2 - 2 * lx) <= 1.0


def test_paper_split_point_figure(golden_dir):
    fig = json.load(open(os.path.join(golden_dir, "fig_split_points.json")))
    fit = json.load(open(os.path.join(golden_dir, "fig_split_ratio.json")))
    v_com = fit["v_com_bytes_per_s"]
    v_gpu = fit["ratio_flop_per_byte_mid"] * v_com
    got = [po.plan_split(po.COST_EQ10, fig["batch"], fig["prompt"] + i, fig["hidden"], fig["elem_bytes"], v_com, v_gpu)[0]
           for i in fig["tokens_generated"]]
    assert got == fig["split_l"]
    # the batch size cancels out of the argmin (every term of Eq. 10 is linear in b)
    got1 = [po.plan_split(po.COST_EQ10, 1, fig["prompt"] + i, fig["hidden"], fig["elem_bytes"], v_com, v_gpu)[0]
            for i in fig["tokens_generated"]]
    assert got1 == fig["split_l"]
    # plausibility of the fitted constants for the paper's machine: ~25 GB/s PCIe 4 and ~250 TFLOP/s
    assert 200e12 < v_gpu < 312e12


def test_granularity_and_latency_terms():
    kw = dict(b=32, s=1000, h=4096, p=2, v_com=57e9, v_gpu=1.2e15)
    l1, t1 = po.plan_split(po.COST_EQ10, **kw)
    l8, t8 = po.plan_split(po.COST_EQ10, granularity=8, **kw)
    assert l8 % 8 == 0 and abs(l8 - l1) < 8 and t8 >= t1
    assert po.candidates(10, 4) == [0, 4, 8, 10]
    assert po.candidates(8, 4) == [0, 4, 8]
    # a fixed latency on each non-empty copy / GEMM: l=0 pays one copy, l=s pays one copy and the GEMM
    t0 = po.cost(po.COST_EQ10, 0, lat_com=1e-3, lat_gpu=5e-4, **kw)
    assert t0 == po.bytes_kv(32, 0, 1000, 4096, 2) / 57e9 + 1e-3
    ts = po.cost(po.COST_EQ10, 1000, lat_com=1e-3, lat_gpu=5e-4, **kw)
    assert ts == (po.bytes_x(32, 1000, 4096, 2) / 57e9 + 1e-3) + (po.flops_recompute(32, 1000, 4096) / 1.2e15 + 5e-4)
    with pytest.raises(ValueError):
        po.candidates(5, 0)


# ---- extension: chunked activation copy -------------------------------------------
def test_chunked_cost_reduces_to_eq10_and_hand_values():
    k = _toy()                                          # t_act = l, t_kv = 2(9-l), t_rc = l
    for l in range(10):
        assert po.cost_chunked(1, l, **k) == po.cost(po.COST_EQ10, l, **k)
    # l = 8, 4 parts: parts land at 2,4,6,8; each GEMM takes 2 -> ends 4,6,8,10; link = 8 + 2 = 10
    assert po.cost_chunked(4, 8, **k) == 10.0
    # l = 9, 3 parts: land 3,6,9; GEMM 3 each -> 6,9,12; link 9 -> 12
    assert po.cost_chunked(3, 9, **k) == 12.0
    # GEMM faster than the link (v_gpu x4): l = 8, 4 parts: GEMM 0.5 each -> last ends 8.5; link 10
    k2 = dict(k, v_gpu=16.0)
    assert po.cost_chunked(4, 8, **k2) == 10.0
    assert po.cost_chunked(4, 9, **k2) == 9.0 + 9.0 / 4 / 4
    # more parts never hurt, and the limit is the link time plus nothing
    real = dict(b=32, s=1024, h=4096, p=2, v_com=57e9, v_gpu=1.0e15)
    ts = [po.plan_split_chunked(c, **real)[1] for c in (1, 2, 4, 8, 16, 32)]
    assert all(a >= b for a, b in zip(ts, ts[1:]))
    assert ts[0] == po.plan_split(po.COST_EQ10, **real)[1]
    assert ts[-1] >= po.bytes_x(32, 1024, 4096, 2) / 57e9


def test_linear_model_reduces_to_the_papers_sizes():
    # with Eq. 6 / Eq. 8 per-position sizes the linear form is Eq. 10 (and its variants) itself
    b, s, h, p = 3, 37, 128, 2
    for model in (po.COST_EQ10, po.COST_NS, po.COST_ROW, po.COST_PIPE):
        for l in range(0, s + 1):
            a = po.cost(model, l, b, s, h, p, 7e9, 3e13, 2e-5, 1e-5)
            c = po.cost_linear(model, 1, l, s, b * h * p, 2 * b * h * p, 4 * b * h * h, 7e9, 3e13, 2e-5, 1e-5)
            assert a == c
        assert po.plan_split(model, b, s, h, p, 7e9, 3e13, 4) == \
            po.plan_split_linear(model, 1, s, b * h * p, 2 * b * h * p, 4 * b * h * h, 7e9, 3e13, 4)
    for chunks in (2, 3, 5):
        for l in (0, 8, 24, 37):
            assert po.cost_chunked(chunks, l, b, s, h, p, 7e9, 3e13, 2e-5, 1e-5) == \
                po.cost_linear(po.COST_EQ10, chunks, l, s, b * h * p, 2 * b * h * p, 4 * b * h * h, 7e9, 3e13, 2e-5, 1e-5)


def test_linear_model_hand_values_with_compressed_sizes():
    # x: 9 B/pos, cache: 18 B/pos, 60 flop/pos, link 3 B/s, GPU 10 flop/s, s = 8
    # l = 2: send_x = 6, gemm = 12, send_kv = 36  -> Eq. 10: 6 + 36 = 42
    # l = 6: send_x = 18, gemm = 36, send_kv = 12 -> Eq. 10: 18 + 36 = 54;  pipe: max(30, 36) = 36
    assert po.cost_linear(po.COST_EQ10, 1, 2, 8, 9, 18, 60, 3.0, 10.0) == 42.0
    assert po.cost_linear(po.COST_EQ10, 1, 6, 8, 9, 18, 60, 3.0, 10.0) == 54.0
    assert po.cost_linear(po.COST_PIPE, 1, 6, 8, 9, 18, 60, 3.0, 10.0) == 36.0
    # crossing of gemm (6 l) and send_kv (6 (8 - l)) is l = 4: t = 12 + 24 = 36, the minimum
    assert po.plan_split_linear(po.COST_EQ10, 1, 8, 9, 18, 60, 3.0, 10.0) == (4, 36.0)


def test_compressing_only_the_cache_disables_recomputation():
    # Sec. 4.4 with the activations left in float16: a position's activations (2h bytes) cost more on the
    # link than its 4-bit cache (9h/8 bytes), so Eq. 10 is increasing in l and l* = 0; with both compressed
    # (9h/16 against 9h/8 bytes) the 1 : 2 ratio of Eq. 6 is back and l* is where it was in float16
    b, s, h = 32, 1024, 4096
    v_com, v_gpu = 57e9, 1.0e15
    fp = 4 * b * h * h
    l_kv_only, _ = po.plan_split_linear(po.COST_EQ10, 1, s, b * 2 * h, b * 9 * h // 8, fp, v_com, v_gpu, 64)
    assert l_kv_only == 0
    l_both, t_both = po.plan_split_linear(po.COST_EQ10, 1, s, b * 9 * h // 16, b * 9 * h // 8, fp, v_com, v_gpu, 1)
    r, k = fp / v_gpu, (b * 9 * h // 8) / v_com
    l_closed = k * s / (r + k)
    assert abs(l_both - l_closed) <= 1
    l_fp16, t_fp16 = po.plan_split(po.COST_EQ10, b, s, h, 2, v_com, v_gpu, 1)
    assert l_both < l_fp16 and t_both < t_fp16       # less to send: the GPU takes a smaller share, the step is shorter


def test_adaptive_estimate_closed_forms():
    # alpha = 1 replaces, alpha = 0 keeps, invalid samples are ignored
    assert po.adapt_update(10.0, 20.0, 1.0, 30, 2.0, 80, 4.0) == (15.0, 20.0)
    assert po.adapt_update(10.0, 20.0, 0.0, 30, 2.0, 80, 4.0) == (10.0, 20.0)
    assert po.adapt_update(10.0, 20.0, 0.5, 0, 2.0, 80, 0.0) == (10.0, 20.0)
    assert po.adapt_update(10.0, 20.0, 0.25, 30, 2.0, 0, 1.0) == (11.25, 20.0)
    # constant observations: the error decays as (1 - alpha)^n
    v, g = 100.0, 7.0
    for n in range(1, 9):
        v, g = po.adapt_update(v, g, 0.5, 40, 1.0, 3, 1.0)
        assert math.isclose(v - 40.0, 60.0 * 0.5 ** n, rel_tol=1e-12)
        assert math.isclose(g - 3.0, 4.0 * 0.5 ** n, rel_tol=1e-12)
    # a link that slows down moves the split towards more recomputation
    l_fast, _ = po.plan_split(po.COST_EQ10, 32, 1024, 4096, 2, 57e9, 1.0e15, 64)
    v2, _ = po.adapt_update(57e9, 1.0e15, 1.0, 300_000_000, 300_000_000 / 28e9, 0, 0.0)
    l_slow, _ = po.plan_split(po.COST_EQ10, 32, 1024, 4096, 2, v2, 1.0e15, 64)
    assert l_slow > l_fast


def test_pipelined_form_with_the_rest_of_the_layer():
    # link 1 B/s, GPU 4 flop/s, b = h = p = 1, s = 9: link(l) = 18 - l, gemm(l) = l; other = 3 -> balance at 18 - l = l + 3
    toy = dict(b=1, s=9, h=1, p=1, v_com=1.0, v_gpu=4.0)
    assert [po.cost(po.COST_PIPE, l, **toy, other=3.0) for l in (0, 7, 8, 9)] == [18.0, 11.0, 11.0, 12.0]
    assert po.plan_split(po.COST_PIPE, **toy, other=3.0) == (7, 11.0)
    assert po.plan_split(po.COST_PIPE, **toy) == (9, 9.0)                 # without it: recompute everything
    # the other forms ignore it
    assert po.cost(po.COST_EQ10, 4, **toy, other=3.0) == po.cost(po.COST_EQ10, 4, **toy)
    assert po.cost_linear(po.COST_PIPE, 1, 7, 9, 1, 2, 4, 1.0, 4.0, other=3.0) == 11.0


def test_recomputation_charged_in_whole_rounds():
    # 60 flop per position, rounds of 100 flop, GPU 10 flop/s: l = 2 -> 120 flop -> 2 rounds = 200 flop = 20 s
    # (link 3 B/s, x 9 B/pos, cache 18 B/pos, s = 8: send_x = 6, send_kv = 36) -> Eq. 10: 6 + max(20, 36) = 42
    assert po.cost_linear(po.COST_EQ10, 1, 2, 8, 9, 18, 60, 3.0, 10.0, round_flops=100) == 42.0
    # l = 6: 360 flop -> 4 rounds = 400 flop = 40 s; send_x = 18, send_kv = 12 -> 18 + 40 = 58 (54 without rounds)
    assert po.cost_linear(po.COST_EQ10, 1, 6, 8, 9, 18, 60, 3.0, 10.0, round_flops=100) == 58.0
    # work that is a whole number of rounds costs the same either way; l = 5 -> 300 flop = 3 rounds
    assert po.cost_linear(po.COST_EQ10, 1, 5, 8, 9, 18, 60, 3.0, 10.0, round_flops=100) == \
        po.cost_linear(po.COST_EQ10, 1, 5, 8, 9, 18, 60, 3.0, 10.0)
    # the plan prefers splits that fill their last round: at the OPT-13B shape (40 tile columns, batch 32) 768
    # positions are 15 full rounds of 256 tiles, 832 are 16.25
    b, h, s = 32, 5120, 1024
    fp, rf = 4 * b * h * h, 256 * 2 * 256 * 256 * h
    v_com, v_gpu = 56e9, 1.10e15
    l_plain, _ = po.plan_split_linear(po.COST_EQ10, 1, s, b * h * 2, 2 * b * h * 2, fp, v_com, v_gpu, 64)
    l_round, t_round = po.plan_split_linear(po.COST_EQ10, 1, s, b * h * 2, 2 * b * h * 2, fp, v_com, v_gpu, 64, round_flops=rf)
    assert (fp * l_round) % rf == 0 or t_round <= po.cost_linear(po.COST_EQ10, 1, l_plain, s, b * h * 2, 2 * b * h * 2, fp, v_com, v_gpu, round_flops=rf)
    assert l_round == 768 and l_plain == 832
