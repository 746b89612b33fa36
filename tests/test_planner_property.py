"""Property test (CPU): for arbitrary per-position sizes, rates, latencies, cost forms, chunk counts and granularities
the library's scheduler returns exactly the oracle's (split, cost): same integer argmin, bit-identical double."""
import pytest
from hypothesis import given, settings, strategies as st

from oracle import kvpr_plan_oracle as po


@pytest.fixture(scope="module")
def k():
    import paper_2411_17089_amd as k
    return k


rates = st.floats(min_value=1e-3, max_value=1e18, allow_nan=False, allow_infinity=False)
lats = st.one_of(st.just(0.0), st.floats(min_value=0.0, max_value=1e-2))
sizes = st.integers(min_value=0, max_value=2 ** 36)


@settings(max_examples=400, deadline=None)
@given(model=st.integers(0, 3), chunks=st.integers(1, 32), s=st.integers(0, 600), x_bpp=sizes, kv_bpp=sizes, fpp=sizes,
       v_com=rates, v_gpu=rates, lat_com=lats, lat_gpu=lats, other=lats, g=st.integers(1, 700),
       rf=st.one_of(st.just(0), st.integers(1, 2 ** 40)))
def test_linear_planner_equals_oracle(k, model, chunks, s, x_bpp, kv_bpp, fpp, v_com, v_gpu, lat_com, lat_gpu, other, g, rf):
    if model != po.COST_EQ10:
        chunks = 1
    prof = k.make_profile(v_com, v_gpu, lat_com, lat_gpu, other, rf)
    want = po.plan_split_linear(model, chunks, s, x_bpp, kv_bpp, fpp, v_com, v_gpu, g, lat_com, lat_gpu, other, rf)
    assert k.kvpr_plan_split_linear(prof, model, chunks, s, x_bpp, kv_bpp, fpp, g) == want
    for l in {0, s // 2, s}:
        assert k.kvpr_cost_linear(prof, model, chunks, l, s, x_bpp, kv_bpp, fpp) == \
            po.cost_linear(model, chunks, l, s, x_bpp, kv_bpp, fpp, v_com, v_gpu, lat_com, lat_gpu, other, rf)


@settings(max_examples=200, deadline=None)
@given(b=st.integers(1, 64), s=st.integers(0, 2048), h=st.sampled_from([64, 768, 4096, 5120, 7168]), v_com=rates, v_gpu=rates,
       model=st.integers(0, 3), g=st.sampled_from([1, 8, 64]))
def test_paper_sizes_planner_equals_oracle(k, b, s, h, v_com, v_gpu, model, g):
    prof = k.make_profile(v_com, v_gpu)
    assert k.kvpr_plan_split(prof, model, b, s, h, 2, g) == po.plan_split(model, b, s, h, 2, v_com, v_gpu, g)
