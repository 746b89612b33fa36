"""CPU-side checks of the C ABI: the library loads, exports every symbol the header
declares, the planner agrees bit for bit with the oracle, and bad arguments are refused
before anything touches the GPU."""
import os
import re

import pytest

from oracle import kvpr_plan_oracle as po

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def k():
    import paper_2411_17089_amd as k
    return k


def test_library_exports_every_declared_symbol(k):
    header = open(os.path.join(ROOT, "include", "kvpr.h")).read()
    declared = set(re.findall(r"\b(kvpr_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(k.EXPORTS), (declared ^ set(k.EXPORTS))
    for name in declared:
        assert hasattr(k.lib, name), name


MODELS = [(po.COST_EQ10, "KVPR_COST_EQ10"), (po.COST_NS, "KVPR_COST_NS"), (po.COST_ROW, "KVPR_COST_ROW"),
          (po.COST_PIPE, "KVPR_COST_PIPE")]


@pytest.mark.parametrize("model,cname", MODELS)
def test_planner_bit_exact_against_oracle(k, model, cname):
    assert getattr(k, cname) == model
    cases = []
    for b in (1, 16, 32, 64):
        for s in (0, 1, 7, 128, 1000, 1024, 4096):
            for h in (768, 4096, 7168):
                for v_com, v_gpu in ((57.3e9, 1.31e15), (32 * 2.0 ** 30, 2.5e14), (1.0, 4.0), (3.3e10, 7.77e14)):
                    cases.append((b, s, h, v_com, v_gpu))
    for b, s, h, v_com, v_gpu in cases:
        prof = k.make_profile(v_com, v_gpu)
        for g in (1, 8):
            want = po.plan_split(model, b, s, h, 2, v_com, v_gpu, granularity=g)
            got = k.kvpr_plan_split(prof, model, b, s, h, 2, g)
            assert got == want, (b, s, h, v_com, v_gpu, g)
        for l in {0, s // 3, s}:
            assert k.kvpr_cost(prof, model, l, b, s, h, 2) == po.cost(model, l, b, s, h, 2, v_com, v_gpu)


def test_planner_ties_and_latency_terms(k):
    prof = k.make_profile(1.0, 4.0)
    assert k.kvpr_plan_split(prof, k.KVPR_COST_NS, 1, 9, 1, 1, 1) == (4, 10.0)     # tie 4/5 -> smallest
    # steady-state form with the rest of the layer's GPU work on the compute arm
    for other in (0.0, 4e-4, 3e-3):
        prof = k.make_profile(57e9, 1.0e15, 0.0, 0.0, other)
        for s in (256, 1024):
            assert k.kvpr_plan_split(prof, k.KVPR_COST_PIPE, 32, s, 4096, 2, 8) == \
                po.plan_split(po.COST_PIPE, 32, s, 4096, 2, 57e9, 1.0e15, 8, 0.0, 0.0, other)
            for l in (0, s // 2, s):
                assert k.kvpr_cost(prof, k.KVPR_COST_PIPE, l, 32, s, 4096, 2) == po.cost(po.COST_PIPE, l, 32, s, 4096, 2, 57e9, 1.0e15, 0.0, 0.0, other)
                assert k.kvpr_cost(prof, k.KVPR_COST_EQ10, l, 32, s, 4096, 2) == po.cost(po.COST_EQ10, l, 32, s, 4096, 2, 57e9, 1.0e15)
    prof = k.make_profile(57e9, 1.2e15, 1e-3, 5e-4)
    for s in (100, 1024):
        want = po.plan_split(po.COST_EQ10, 32, s, 4096, 2, 57e9, 1.2e15, 1, 1e-3, 5e-4)
        assert k.kvpr_plan_split(prof, k.KVPR_COST_EQ10, 32, s, 4096, 2, 1) == want
        for l in (0, 1, s):
            assert k.kvpr_cost(prof, 0, l, 32, s, 4096, 2) == po.cost(0, l, 32, s, 4096, 2, 57e9, 1.2e15, 1e-3, 5e-4)


def test_chunked_planner_bit_exact_against_oracle(k):
    for b, s, h, v_com, v_gpu in [(32, 1024, 4096, 57.3e9, 1.05e15), (1, 128, 768, 20e9, 3e13), (16, 4096, 7168, 55e9, 9e14),
                                  (4, 37, 256, 1e9, 5e11)]:
        for lat in ((0.0, 0.0), (2e-5, 1e-5)):
            prof = k.make_profile(v_com, v_gpu, *lat)
            for chunks in (1, 2, 5, 8, 32):
                for g in (1, 8):
                    want = po.plan_split_chunked(chunks, b, s, h, 2, v_com, v_gpu, g, *lat)
                    assert k.kvpr_plan_split_chunked(prof, chunks, b, s, h, 2, g) == want
                for l in {0, 1, s // 2, s}:
                    assert k.kvpr_cost_chunked(prof, chunks, l, b, s, h, 2) == po.cost_chunked(chunks, l, b, s, h, 2, v_com, v_gpu, *lat)
            for l in {0, s // 3, s}:
                assert k.kvpr_cost_chunked(prof, 1, l, b, s, h, 2) == k.kvpr_cost(prof, k.KVPR_COST_EQ10, l, b, s, h, 2)
    with pytest.raises(k.KvprError) as e:
        k.kvpr_plan_split_chunked(k.make_profile(1e9, 1e12), 0, 1, 8, 64, 2, 1)
    assert e.value.code == k.KVPR_E_RANGE


def test_linear_planner_bit_exact_against_oracle(k):
    """Per-position sizes (Eq. 6 / Eq. 8 as rates): the paper's, and those of a 4-bit store (Sec. 4.4)."""
    from oracle import kvpr_int4_oracle as qo
    for b, s, h, v_com, v_gpu in [(32, 1024, 4096, 57.3e9, 1.05e15), (1, 128, 768, 20e9, 3e13), (16, 4096, 7168, 55e9, 9e14),
                                  (4, 37, 256, 1e9, 5e11)]:
        sizes = [(b * h * 2, 2 * b * h * 2), (b * qo.packed_bytes(h), b * qo.packed_bytes(2 * h)),
                 (b * h * 2, b * qo.packed_bytes(2 * h)), (0, 17)]
        assert k.kvpr_int4_row_bytes(h) == qo.packed_bytes(h) and k.kvpr_int4_row_bytes(2 * h) == qo.packed_bytes(2 * h)
        fp = 4 * b * h * h
        for lat in ((0.0, 0.0), (2e-5, 1e-5)):
            prof = k.make_profile(v_com, v_gpu, *lat)
            for xb, kb in sizes:
                for model, _ in MODELS:
                    for chunks in ((1, 3) if model == po.COST_EQ10 else (1,)):
                        for g in (1, 8):
                            want = po.plan_split_linear(model, chunks, s, xb, kb, fp, v_com, v_gpu, g, *lat)
                            assert k.kvpr_plan_split_linear(prof, model, chunks, s, xb, kb, fp, g) == want
                        for l in {0, 1, s // 2, s}:
                            assert k.kvpr_cost_linear(prof, model, chunks, l, s, xb, kb, fp) == \
                                po.cost_linear(model, chunks, l, s, xb, kb, fp, v_com, v_gpu, *lat)
            # the paper's sizes through the linear entry point are kvpr_plan_split itself
            assert k.kvpr_plan_split_linear(prof, 0, 1, s, b * h * 2, 2 * b * h * 2, fp, 1) == k.kvpr_plan_split(prof, 0, b, s, h, 2, 1)
    good = k.make_profile(1e9, 1e12)
    for args, code in (((0, 1, 8, -1, 4, 4, 1), k.KVPR_E_RANGE), ((0, 0, 8, 2, 4, 4, 1), k.KVPR_E_RANGE),
                       ((1, 2, 8, 2, 4, 4, 1), k.KVPR_E_INVAL), ((0, 1, 8, 2, 4, 4, 0), k.KVPR_E_RANGE),
                       ((0, 1, 8, 2 ** 60, 4, 4, 1), k.KVPR_E_RANGE)):
        with pytest.raises(k.KvprError) as e:
            k.kvpr_plan_split_linear(good, *args)
        assert e.value.code == code, args
    assert k.kvpr_int4_row_bytes(100) == 0 and k.kvpr_int4_row_bytes(0) == 0


def test_adaptive_update_bit_exact_against_oracle(k):
    import random
    rnd = random.Random(5)
    for _ in range(300):
        v_com, v_gpu = rnd.uniform(1e9, 9e10), rnd.uniform(1e13, 2e15)
        alpha = rnd.choice([0.0, 1.0, 0.5, rnd.random()])
        lb, ls = rnd.choice([0, rnd.randrange(1, 10 ** 10)]), rnd.choice([0.0, rnd.uniform(1e-5, 1e-1)])
        fl, gs = rnd.choice([0, rnd.randrange(1, 10 ** 13)]), rnd.choice([0.0, rnd.uniform(1e-5, 1e-2)])
        prof = k.kvpr_adapt_update(k.make_profile(v_com, v_gpu), alpha, lb, ls, fl, gs)
        assert (prof.h2d_bytes_per_s, prof.gemm_flops_per_s) == po.adapt_update(v_com, v_gpu, alpha, lb, ls, fl, gs)
    for alpha in (-0.1, 1.5, float("nan")):
        with pytest.raises(k.KvprError) as e:
            k.kvpr_adapt_update(k.make_profile(1e9, 1e12), alpha, 1, 1.0, 1, 1.0)
        assert e.value.code == k.KVPR_E_RANGE


def test_rotary_table_against_oracle(k):
    from oracle import kvpr_llama_oracle as lo
    import numpy as np
    for d, base in ((64, 10000.0), (128, 10000.0), (128, 500000.0)):
        t = k.kvpr_rope_table(300, d, base)
        ang = lo.rope_angles(np.arange(300), d, base)
        assert t.shape == (300, d // 2, 2)
        assert np.abs(t[..., 0] - np.cos(ang)).max() <= 1.3e-7 and np.abs(t[..., 1] - np.sin(ang)).max() <= 1.3e-7
    for args, code in (((10, 96, 10000.0), k.KVPR_E_RANGE), ((0, 64, 10000.0), k.KVPR_E_RANGE), ((4, 64, 0.0), k.KVPR_E_INVAL)):
        with pytest.raises(k.KvprError) as e:
            k.kvpr_rope_table(*args)
        assert e.value.code == code


def test_planner_rejects_bad_arguments(k):
    good = k.make_profile(1e9, 1e12)
    for prof in (k.make_profile(0.0, 1e12), k.make_profile(1e9, -1.0), k.make_profile(float("nan"), 1e12),
                 k.make_profile(1e9, float("inf")), k.make_profile(1e9, 1e12, -1.0, 0.0)):
        with pytest.raises(k.KvprError) as e:
            k.kvpr_plan_split(prof, 0, 1, 8, 64, 2, 1)
        assert e.value.code == k.KVPR_E_INVAL
    for args in ((7, 1, 8, 64, 2, 1),):
        with pytest.raises(k.KvprError) as e:
            k.kvpr_plan_split(good, *args)
        assert e.value.code == k.KVPR_E_INVAL
    for args in ((0, 0, 8, 64, 2, 1), (0, 1, -1, 64, 2, 1), (0, 1, 8, 64, 2, 0), (0, 1, 8, 0, 2, 1)):
        with pytest.raises(k.KvprError) as e:
            k.kvpr_plan_split(good, *args)
        assert e.value.code == k.KVPR_E_RANGE
    with pytest.raises(k.KvprError) as e:
        k.kvpr_cost(good, 0, 9, 1, 8, 64, 2)
    assert e.value.code == k.KVPR_E_RANGE
    assert "split" in k.kvpr_last_error()


def test_kernel_entry_points_validate_before_touching_the_gpu(k):
    with pytest.raises(k.KvprError) as e:
        k.kvpr_recompute_gemm(1, 1, None, 1, 5, 64, 100, 64, stream=0)       # K % 64
    assert e.value.code == k.KVPR_E_INVAL
    with pytest.raises(k.KvprError) as e:
        k.kvpr_recompute_gemm(1, 1, None, 1, -1, 64, 64, 64, stream=0)
    assert e.value.code == k.KVPR_E_RANGE
    with pytest.raises(k.KvprError) as e:
        k.kvpr_decode_attention(1, 1, 1, 1, 4, 1, 96, 1, stream=0)            # head_dim 96
    assert e.value.code == k.KVPR_E_INVAL
    with pytest.raises(k.KvprError) as e:
        k.kvpr_decode_attention(1, 1, 1, 1, 0, 1, 128, 1, stream=0)           # S = 0
    assert e.value.code == k.KVPR_E_RANGE
    with pytest.raises(k.KvprError) as e:
        k.kvpr_token_gemm(1, 1, None, 1, 1, 65, 64, 128, 0, 64, stream=0)     # M > 64
    assert e.value.code == k.KVPR_E_RANGE
    assert k.kvpr_attention_workspace_bytes(32, 4096, 32, 1025) > 0
    # token GEMM workspace: 4096 bytes of arrival counters + 8 K slices of float32 partial tiles, N rounded up to whole
    # blocks of 128 features, M to whole tiles of 16 rows
    assert k.kvpr_token_gemm_workspace_bytes(32, 7168) == 4096 + 8 * 7168 * 32 * 4
    assert k.kvpr_token_gemm_workspace_bytes(33, 100) == 4096 + 8 * 128 * 48 * 4
    assert k.kvpr_token_gemm_workspace_bytes(0, 128) == 0 and k.kvpr_token_gemm_workspace_bytes(65, 128) == 0
    assert k.kvpr_token_gemm_workspace_bytes(1, 0) == 0
    with pytest.raises(k.KvprError) as e:
        k.kvpr_token_gemm_ws(1, 1, None, 1, 1, 32, 64, 100, 0, 64, 16, 8192, stream=0)   # K % 128
    assert e.value.code == k.KVPR_E_INVAL
    with pytest.raises(k.KvprError) as e:
        k.kvpr_token_gemm_ws(1, 1, None, 1, 1, 32, 64, 128, 0, 64, 8, 8192, stream=0)    # workspace not 16-byte aligned
    assert e.value.code == k.KVPR_E_INVAL
    for fn in (k.kvpr_quant_int4, k.kvpr_dequant_int4):
        with pytest.raises(k.KvprError) as e:
            fn(1, 1, 4, 100, stream=0)                                         # cols % 64
        assert e.value.code == k.KVPR_E_RANGE
        with pytest.raises(k.KvprError) as e:
            fn(None, 1, 4, 128, stream=0)
        assert e.value.code == k.KVPR_E_INVAL


def test_create_rejects_bad_descriptions(k):
    bad = [dict(hidden=768, n_heads=12, head_dim=32), dict(hidden=768, n_heads=11, head_dim=64),
           dict(hidden=96 * 2, n_heads=2, head_dim=96), dict(dtype=7), dict(dtype=0x100), dict(dtype=0x401), dict(ffn_dim=100), dict(arch=2),
           dict(arch=1, rope_base=-1.0)]
    base = dict(n_layers=1, hidden=768, n_heads=12, head_dim=64, ffn_dim=0, batch=1, max_seq=16, dtype=k.KVPR_F16)
    for upd in bad:
        kw = dict(base, **upd)
        with pytest.raises(k.KvprError) as e:
            k.kvpr_create(stream=0, **kw)
        assert e.value.code == k.KVPR_E_INVAL, upd
    for upd in (dict(batch=0), dict(n_layers=0), dict(max_seq=0), dict(batch=65)):
        with pytest.raises(k.KvprError) as e:
            k.kvpr_create(stream=0, **dict(base, **upd))
        assert e.value.code == k.KVPR_E_RANGE, upd
