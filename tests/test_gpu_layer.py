"""GPU parity of kvpr_layer_decode against the CPU oracle: every split of the small config,
split invariance on the device, debug modes, store-back, and argument checks that need a context."""
import ctypes

import numpy as np
import pytest
import torch

import kvpr_inputs
from oracle import kvpr_oracle as ko
from kvpr_testlib import dev, rel_err, rel_err_rms, upload_layer

pytestmark = pytest.mark.gpu
TOL = 1e-2
TIGHT = 3e-3


@pytest.fixture(scope="module")
def k():
    import paper_2411_17089_amd as k
    return k


class Rig:
    """One attention layer on the device plus its oracle-side data."""

    def __init__(self, k, seed, b, s, h, H, max_seq=None, n_layers=1):
        self.k, self.b, self.s, self.h, self.H = k, b, s, h, H
        self.layer = kvpr_inputs.make_layer(seed, b, s, h, H)
        self.stored = ko.stored_kv(self.layer, "fp16")                     # what prefill left on the host
        self.d = upload_layer(self.layer)
        self.w = k.make_weights(wqkv=self.d["wqkv"], bqkv=self.d["bqkv"], wo=self.d["wo"], bo=self.d["bo"])
        self.ctx = k.kvpr_create(n_layers, h, H, h // H, 0, b, max_seq or s + 2)
        for layer in range(n_layers):
            k.kvpr_store_write(self.ctx, layer, 0, s, np.ascontiguousarray(self.layer["X"]),
                               np.ascontiguousarray(self.stored.astype(np.float16)))
        self.out = torch.empty((b, h), dtype=torch.float16, device="cuda")

    def decode(self, l, layer=0, timing=False):
        t = self.k.kvpr_layer_decode(self.ctx, layer, self.s, l, self.w, self.d["x_new"], self.out, timing)
        torch.cuda.synchronize()
        return self.out.cpu().numpy().copy(), t

    def host_rows(self, layer=0):
        xp, kvp = self.k.kvpr_store_ptrs(self.ctx, layer)
        n_x, n_kv = (self.s + 1) * self.b * self.h, (self.s + 1) * self.b * 2 * self.h
        x = np.ctypeslib.as_array(ctypes.cast(xp, ctypes.POINTER(ctypes.c_uint16)), (n_x,)).view(np.float16)
        kv = np.ctypeslib.as_array(ctypes.cast(kvp, ctypes.POINTER(ctypes.c_uint16)), (n_kv,)).view(np.float16)
        return x.reshape(self.s + 1, self.b, self.h), kv.reshape(self.s + 1, self.b, 2 * self.h)

    def close(self):
        self.k.kvpr_destroy(self.ctx)


def test_small_config_every_split(k):
    """hidden 768, 12 heads x 64, batch 1, context 128: all 129 splits against the oracle."""
    rig = Rig(k, 0, 1, 128, 768, 12)
    try:
        ref = ko.layer_decode(rig.layer, 0, rig.stored)["o"]
        outs = []
        for l in range(129):
            print(f"small config split {l}", flush=True)
            o, _ = rig.decode(l)
            outs.append(o)
            assert rel_err(o, ref) <= TIGHT, l
            assert rel_err_rms(o, ref) <= TOL, l
        # on the device the recomputed rows may differ from the transferred ones by fp16 rounding of an
        # fp32 (not fp64) sum, so outputs at different splits agree to rounding, not bit for bit
        spread = max(rel_err(o, outs[0]) for o in outs)
        assert spread <= 2e-3
    finally:
        rig.close()


@pytest.mark.parametrize("seed,b,s,h,H", [(1, 3, 77, 256, 2), (2, 32, 40, 512, 4), (3, 5, 300, 768, 12), (4, 2, 1, 128, 1),
                                          (5, 33, 20, 256, 4)])
def test_layer_decode_shapes(k, seed, b, s, h, H):
    rig = Rig(k, seed, b, s, h, H)
    try:
        ref = ko.layer_decode(rig.layer, 0, rig.stored)
        for l in sorted({0, 1, s // 2, s - 1, s} & set(range(s + 1))):
            print(f"layer decode b={b} s={s} h={h} H={H} split={l}", flush=True)
            o, _ = rig.decode(l)
            assert rel_err(o, ref["o"]) <= TIGHT, l
        # store-back: row s of the host store now holds x_new and the new K|V row (Eq. 5)
        x_host, kv_host = rig.host_rows()
        assert np.array_equal(x_host[s], rig.layer["x_new"])
        assert rel_err(kv_host[s], ref["kv"][s]) <= 1e-3
        assert np.array_equal(x_host[:s], rig.layer["X"])
    finally:
        rig.close()


def test_seq_zero_is_attention_over_the_new_token_only(k):
    rig = Rig(k, 6, 2, 0, 256, 2, max_seq=4)
    try:
        o, _ = rig.decode(0)
        ref = ko.layer_decode(rig.layer, 0, rig.stored)["o"]
        assert rel_err(o, ref) <= TIGHT
    finally:
        rig.close()


def test_debug_modes_do_not_change_the_result(k):
    rig = Rig(k, 7, 4, 90, 512, 4)
    try:
        base, _ = rig.decode(37)
        for flags in (k.KVPR_DEBUG_SYNC, k.KVPR_DEBUG_POISON, k.KVPR_DEBUG_SYNC | k.KVPR_DEBUG_POISON):
            k.kvpr_set_debug(rig.ctx, flags)
            o, _ = rig.decode(37)
            assert np.array_equal(o, base), flags         # a missed fence would leave NaN poison in the cache
            assert np.isfinite(o).all()
        k.kvpr_set_debug(rig.ctx, 0)
        for l in (0, 90):
            k.kvpr_set_debug(rig.ctx, k.KVPR_DEBUG_POISON)
            o, _ = rig.decode(l)
            assert np.isfinite(o).all(), l
    finally:
        rig.close()


def test_timing_and_planned_split(k):
    rig = Rig(k, 8, 8, 200, 1024, 8)
    try:
        prof = k.make_profile(50e9, 4e14)
        k.kvpr_set_profile(rig.ctx, prof, k.KVPR_COST_EQ10, 1)
        want_l, want_t = k.kvpr_plan_split(prof, k.KVPR_COST_EQ10, 8, 200, 1024, 2, 1)
        o, t = rig.decode(-1, timing=True)
        assert t.split == want_l and t.t_bound_s == want_t
        assert t.ms_total > 0 and t.ms_assemble > 0 and t.ms_total >= t.ms_assemble
        assert t.ms_attn > 0 and t.ms_proj > 0
        assert rel_err(o, ko.layer_decode(rig.layer, 0, rig.stored)["o"]) <= TIGHT
    finally:
        rig.close()


def test_context_argument_checks(k):
    rig = Rig(k, 9, 2, 10, 256, 2, max_seq=12)
    try:
        cases = [
            (dict(seq=12), k.KVPR_E_RANGE),       # seq + 1 > max_seq
            (dict(split=11), k.KVPR_E_RANGE),     # split > seq
            (dict(split=-2), k.KVPR_E_RANGE),
            (dict(layer=1), k.KVPR_E_RANGE),
            (dict(split=-1), k.KVPR_E_STATE),     # no profile set
            (dict(seq=11, split=11), k.KVPR_E_STATE),   # row 10 never written
        ]
        for upd, code in cases:
            kw = dict(layer=0, seq=10, split=3)
            kw.update(upd)
            with pytest.raises(k.KvprError) as e:
                k.kvpr_layer_decode(rig.ctx, kw["layer"], kw["seq"], kw["split"], rig.w, rig.d["x_new"], rig.out)
            assert e.value.code == code, (upd, str(e.value))
        with pytest.raises(k.KvprError):
            k.kvpr_layer_decode(rig.ctx, 0, 10, 3, rig.w, None, rig.out)
        with pytest.raises(k.KvprError):
            k.kvpr_store_write(rig.ctx, 0, 5, 13, None, None)
        # after one decode at seq=10 the store holds row 10, so seq=11 becomes legal... but needs max_seq >= 12: ok
        rig.decode(4)
        k.kvpr_layer_decode(rig.ctx, 0, 11, 11, rig.w, rig.d["x_new"], rig.out)
        torch.cuda.synchronize()
    finally:
        rig.close()


def test_two_decode_steps_grow_the_cache(k):
    """Generate two tokens: the second step must see the first step's stored-back row."""
    b, s, h, H = 2, 30, 256, 2
    rig = Rig(k, 10, b, s, h, H, max_seq=s + 3)
    try:
        o1, _ = rig.decode(12)
        x2 = kvpr_inputs._draw(np.random.default_rng(99), (b, h), 1.0)
        layer2 = dict(rig.layer)
        layer2["X"] = np.concatenate([rig.layer["X"], rig.layer["x_new"][None]], 0)
        layer2["x_new"] = x2
        ref2 = ko.layer_decode(layer2, 0)["o"]
        out2 = torch.empty((b, h), dtype=torch.float16, device="cuda")
        for l in (0, 31, 17):
            k.kvpr_layer_decode(rig.ctx, 0, s + 1, l, rig.w, dev(x2), out2)
            torch.cuda.synchronize()
            assert rel_err(out2.cpu().numpy(), ref2) <= TIGHT, l
    finally:
        rig.close()


def test_prefill_helper_matches_oracle_cache(k):
    rig = Rig(k, 11, 4, 50, 512, 4)
    try:
        k.kvpr_store_write(rig.ctx, 0, 0, 50, None, np.zeros((50, 4, 1024), np.float16))
        k.kvpr_store_prefill_kv(rig.ctx, 0, 50, rig.w)
        _, kv_host = rig.host_rows()
        assert rel_err(kv_host[:50], rig.stored) <= 1e-3
        assert np.mean(kv_host[:50].astype(np.float64) != rig.stored) < 0.05
    finally:
        rig.close()


def test_chunked_activation_copy_gives_identical_results(k):
    """Extension: X[0:l] copied in parts with the GEMM of each part started as it lands.  Row results of
    the GEMM do not depend on how rows are grouped into launches, so outputs must be bit-identical."""
    rig = Rig(k, 12, 32, 200, 512, 4)
    try:
        for l in (0, 5, 64, 133, 200):
            base, _ = rig.decode(l)
            for chunks in (2, 3, 8, 32):
                k.kvpr_set_chunks(rig.ctx, chunks)
                k.kvpr_set_debug(rig.ctx, k.KVPR_DEBUG_POISON)
                o, t = rig.decode(l, timing=True)
                assert np.array_equal(o, base), (l, chunks)
                assert t.split == l
                k.kvpr_set_debug(rig.ctx, 0)
                k.kvpr_set_chunks(rig.ctx, 1)
        ref = ko.layer_decode(rig.layer, 0, rig.stored)["o"]
        assert rel_err(base, ref) <= TIGHT
        with pytest.raises(k.KvprError):
            k.kvpr_set_chunks(rig.ctx, 33)
        # planned split follows the chunked model when chunks > 1
        prof = k.make_profile(50e9, 4e14)
        k.kvpr_set_profile(rig.ctx, prof, k.KVPR_COST_EQ10, 8)
        k.kvpr_set_chunks(rig.ctx, 4)
        o, t = rig.decode(-1, timing=True)
        want_l, want_t = k.kvpr_plan_split_chunked(prof, 4, 32, 200, 512, 2, 8)
        assert t.split == want_l and t.t_bound_s == k.kvpr_cost_chunked(prof, 4, want_l, 32, 200, 512, 2)
        assert rel_err(o, ref) <= TIGHT
    finally:
        rig.close()


def test_batch_64_and_head_dim_64(k):
    """Largest supported batch (four 16-row MFMA tiles in the token GEMM) with 64-wide heads."""
    rig = Rig(k, 13, 64, 24, 256, 4)
    try:
        ref = ko.layer_decode(rig.layer, 0, rig.stored)["o"]
        for l in (0, 11, 24):
            o, _ = rig.decode(l)
            assert rel_err(o, ref) <= TIGHT, l
    finally:
        rig.close()


def test_profile_reports_sane_rates(k):
    ctx = k.kvpr_create(1, 1024, 8, 128, 0, 8, 300)
    try:
        p = k.kvpr_profile(ctx, 8, 256)
        assert 1e9 < p.h2d_bytes_per_s < 1e11 and 1e9 < p.d2h_bytes_per_s < 1e11
        assert p.h2d_peak_bytes_per_s >= p.h2d_bytes_per_s * 0.999
        assert 1e12 < p.gemm_flops_per_s < 2.6e15
        assert 1e10 < p.attn_bytes_per_s < 8.5e12
        assert p.h2d_latency_s == 0.0 and p.gemm_latency_s == 0.0
        assert 2e-6 < p.layer_other_s < 5e-3                   # projections + attention of a small layer
        k.kvpr_set_profile(ctx, p, k.KVPR_COST_EQ10, 1)
        with pytest.raises(k.KvprError) as e:
            k.kvpr_profile(ctx, 8, 300)                      # batch*seq beyond the context
        assert e.value.code == k.KVPR_E_RANGE
    finally:
        k.kvpr_destroy(ctx)
    # a full decoder layer (both FFN kinds): the FFN is part of the rest-of-layer time
    for arch, ffn in ((k.KVPR_ARCH_OPT, 4096), (k.KVPR_ARCH_LLAMA, 2816)):
        ctx = k.kvpr_create(2, 1024, 8, 128, ffn, 8, 300, arch=arch)
        try:
            p2 = k.kvpr_profile(ctx, 8, 256)
            assert p2.layer_other_s > p.layer_other_s * 0.8 and p2.layer_other_s < 5e-3
        finally:
            k.kvpr_destroy(ctx)


def test_profile_step_refines_only_the_gemm_rate(k):
    """The step rehearsal replaces v_gpu by a sane figure, leaves every other field alone, works with and without the
    clock keep-alive, on both architectures and on a packed store, and refuses what it cannot measure."""
    import ctypes
    for arch, flags in ((k.KVPR_ARCH_OPT, 0), (k.KVPR_ARCH_LLAMA, 0), (k.KVPR_ARCH_OPT, k.KVPR_KV_INT4 | k.KVPR_X_INT4),
                        (k.KVPR_ARCH_OPT, k.KVPR_KV_INT4)):     # cache-only packing: X rows are the larger ones
        ctx = k.kvpr_create(1, 1024, 8, 128, 0, 16, 1026, dtype=k.KVPR_F16 | flags, arch=arch)
        try:
            p = k.kvpr_profile(ctx, 16, 1024)
            for frac in (0.0, 0.85):
                k.kvpr_set_keep_warm(ctx, frac)
                q = k.kvpr_profile_step(ctx, 16, 1024, p)
                assert 0.3 * p.gemm_flops_per_s < q.gemm_flops_per_s < 2.6e15
                a, b_ = bytearray(bytes(p)), bytearray(bytes(q))
                off = type(p).gemm_flops_per_s.offset
                a[off:off + 8] = b_[off:off + 8] = bytes(8)
                assert a == b_
            q = k.kvpr_profile_step(ctx, 3, 40, p)                   # below one granule: rehearsed at l = seq
            assert 1e11 < q.gemm_flops_per_s < 2.6e15
            for bad in ((17, 64), (16, 1026), (0, 64), (16, 0)):
                with pytest.raises(k.KvprError) as e:
                    k.kvpr_profile_step(ctx, bad[0], bad[1], p)
                assert e.value.code == k.KVPR_E_RANGE
            with pytest.raises(k.KvprError) as e:
                k.kvpr_profile_step(ctx, 16, 1024, k.make_profile(0.0, 1e12))
            assert e.value.code == k.KVPR_E_INVAL
        finally:
            k.kvpr_destroy(ctx)


def test_adaptive_profile_tracks_the_measured_rates(k):
    """Start from a profile whose link rate is 3x too high: untimed decodes record probes, the planner folds them in
    and the estimate converges to what the copies actually achieve; results stay correct throughout."""
    from oracle import kvpr_plan_oracle as po
    b, s, h, H = 16, 512, 1024, 8
    rig = Rig(k, 31, b, s, h, H)
    try:
        ref = ko.layer_decode(rig.layer, 0, rig.stored)["o"]
        true = k.kvpr_profile(rig.ctx, b, s)
        wrong = k.make_profile(3.0 * true.h2d_bytes_per_s, true.gemm_flops_per_s)
        sizes = (b * h * 2, 2 * b * h * 2, 4 * b * h * h)
        k.kvpr_set_profile(rig.ctx, wrong, k.KVPR_COST_EQ10, 8)
        l_wrong, _ = k.kvpr_plan_split_linear(wrong, k.KVPR_COST_EQ10, 1, s, *sizes, 8)
        # alpha = 0: nothing moves
        for _ in range(3):
            o, _ = rig.decode(-1)
        got = k.kvpr_get_profile(rig.ctx)
        assert got.h2d_bytes_per_s == wrong.h2d_bytes_per_s and got.gemm_flops_per_s == wrong.gemm_flops_per_s
        k.kvpr_set_adaptive(rig.ctx, 0.5)
        for i in range(14):
            print(f"adaptive decode {i}", flush=True)
            o, _ = rig.decode(-1)
            assert rel_err(o, ref) <= TIGHT
        got = k.kvpr_get_profile(rig.ctx)
        print("link GB/s: wrong %.1f adapted %.1f profiler %.1f; gemm TF: adapted %.0f profiler %.0f" % (
            wrong.h2d_bytes_per_s / 1e9, got.h2d_bytes_per_s / 1e9, true.h2d_bytes_per_s / 1e9,
            got.gemm_flops_per_s / 1e12, true.gemm_flops_per_s / 1e12), flush=True)
        assert got.h2d_bytes_per_s < 1.6 * true.h2d_bytes_per_s          # came down from 3x
        assert got.h2d_bytes_per_s > 0.3 * true.h2d_bytes_per_s
        assert 0.2 * true.gemm_flops_per_s < got.gemm_flops_per_s < 3.0 * true.gemm_flops_per_s
        l_now, _ = k.kvpr_plan_split_linear(got, k.KVPR_COST_EQ10, 1, s, *sizes, 8)
        want, _ = po.plan_split_linear(po.COST_EQ10, 1, s, *sizes, got.h2d_bytes_per_s, got.gemm_flops_per_s, 8)
        assert l_now == want and l_now > l_wrong                          # a slower link: recompute more
        with pytest.raises(k.KvprError) as e:
            k.kvpr_set_adaptive(rig.ctx, 1.5)
        assert e.value.code == k.KVPR_E_RANGE
    finally:
        rig.close()


def test_keep_warm_changes_timing_but_not_results(k):
    """The clock keep-alive puts a wall-time-bounded MFMA loop in front of the recompute GEMM: outputs are bit for bit
    those without it, the GEMM starts no earlier than the requested busy time, and the loop ends by itself."""
    rig = Rig(k, 21, 8, 512, 1024, 8)
    try:
        l = 384
        base, _ = rig.decode(l)
        assert rel_err(base, ko.layer_decode(rig.layer, l, rig.stored)["o"]) <= TIGHT
        # a profile that claims a slow link (10 GB/s): X[0:384] = 6 MiB then "takes" 0.63 ms, of which 0.9 are kept busy
        prof = k.make_profile(10e9, 1e15)
        k.kvpr_set_profile(rig.ctx, prof, k.KVPR_COST_EQ10, 1)
        # one-time costs (kernel loading, first touch) put multi-millisecond outliers into the first decodes of a process:
        # every figure is the smallest of a few repeats
        start_off = min(rig.decode(l, timing=True)[1].ms_recompute_start for _ in range(4))
        k.kvpr_set_keep_warm(rig.ctx, 0.9)
        starts = []
        for rep in range(4):
            print(f"keep-warm decode {rep}", flush=True)
            got, t_on = rig.decode(l, timing=True)
            assert np.array_equal(got, base)
            starts.append(t_on.ms_recompute_start)
        want_ms = 0.9 * l * 8 * 1024 * 2 / 10e9 * 1e3
        print(f"recompute could start at {start_off:.3f} ms without, {min(starts):.3f} ms with (all: {starts}; "
              f"requested busy time {want_ms:.3f} ms)", flush=True)
        assert min(starts) >= want_ms                            # never earlier than asked
        assert min(starts) <= want_ms + 0.5                      # the loop is bounded by wall time: it ended about when asked
        k.kvpr_set_keep_warm(rig.ctx, 0.0)
        back = []
        for rep in range(3):
            got, t_back = rig.decode(l, timing=True)
            assert np.array_equal(got, base)
            back.append(t_back.ms_recompute_start)
        assert min(back) < want_ms
        with pytest.raises(k.KvprError):
            k.kvpr_set_keep_warm(rig.ctx, 1.5)
    finally:
        rig.close()
