"""GPU parity of kvpr_decode_step (layer-pipelined decode through a stack of decoder layers)
against the CPU oracle."""
import ctypes

import numpy as np
import pytest
import torch

import kvpr_inputs
from oracle import kvpr_oracle as ko
from kvpr_testlib import dev, rel_err, upload_layer

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def k():
    import paper_2411_17089_amd as k
    return k


class Stack:
    def __init__(self, k, n_layers, b, s, h, H, ffn, max_seq=None, seed0=100):
        self.k, self.n, self.b, self.s, self.h = k, n_layers, b, s, h
        self.layers = []
        for i in range(n_layers):
            L = kvpr_inputs.make_layer(seed0 + i, b, s, h, H)
            L.update(kvpr_inputs.make_ffn(seed0 + i, h, ffn))
            self.layers.append(L)
        self.stored = [ko.stored_kv(L, "fp16") for L in self.layers]
        self.dev = [upload_layer(L) for L in self.layers]
        self.w = [k.make_weights(**{f: d[f] for f in ("wqkv", "bqkv", "wo", "bo", "ln1_g", "ln1_b", "w1", "b1", "w2", "b2",
                                                      "ln2_g", "ln2_b")}) for d in self.dev]
        self.ctx = k.kvpr_create(n_layers, h, H, h // H, ffn, b, max_seq or s + 3)
        for i, L in enumerate(self.layers):
            k.kvpr_store_write(self.ctx, i, 0, s, np.ascontiguousarray(L["X"]), self.stored[i].astype(np.float16))
        self.x_in = kvpr_inputs._draw(np.random.default_rng(seed0 - 1), (b, h), 1.0)
        self.x_out = torch.empty((b, h), dtype=torch.float16, device="cuda")

    def close(self):
        self.k.kvpr_destroy(self.ctx)


@pytest.mark.parametrize("n_layers,b,s,h,H,ffn", [(3, 4, 48, 256, 2, 1024), (5, 2, 33, 768, 12, 3072), (2, 32, 20, 512, 4, 2048)])
def test_decode_step_matches_oracle(k, n_layers, b, s, h, H, ffn):
    st = Stack(k, n_layers, b, s, h, H, ffn)
    try:
        rng = np.random.default_rng(7)
        for trial in range(3):
            splits = [int(v) for v in rng.integers(0, s + 1, n_layers)]
            if trial == 0:
                splits = [0] * n_layers
            if trial == 1:
                splits = [s] * n_layers
            print(f"decode_step layers={n_layers} b={b} s={s} h={h} splits={splits}", flush=True)
            got_splits, _ = k.kvpr_decode_step(st.ctx, s, st.w, dev(st.x_in), st.x_out, splits)
            torch.cuda.synchronize()
            assert got_splits == splits
            ref, trace = ko.decoder_stack_decode(st.layers, st.x_in, splits, st.stored)
            got = st.x_out.cpu().numpy()
            assert rel_err(got, ref) <= 1e-2
            assert rel_err(got, ref) <= 5e-3
        # store-back of every layer: row s holds that layer's post-LayerNorm input and new K|V row
        for i in range(n_layers):
            xp, kvp = k.kvpr_store_ptrs(st.ctx, i)
            x_host = np.ctypeslib.as_array(ctypes.cast(xp, ctypes.POINTER(ctypes.c_uint16)), ((s + 1) * b * h,)).view(np.float16).reshape(s + 1, b, h)
            kv_host = np.ctypeslib.as_array(ctypes.cast(kvp, ctypes.POINTER(ctypes.c_uint16)), ((s + 1) * b * 2 * h,)).view(np.float16).reshape(s + 1, b, 2 * h)
            assert rel_err(x_host[s], trace[i]["xn"]) <= 3e-3, i
            assert rel_err(kv_host[s], trace[i]["kv_new"]) <= 5e-3, i
    finally:
        st.close()


def test_decode_step_planned_splits_timing_and_debug(k):
    st = Stack(k, 4, 4, 64, 256, 2, 1024)
    try:
        prof = k.make_profile(40e9, 2e14)
        k.kvpr_set_profile(st.ctx, prof, k.KVPR_COST_EQ10, 1)
        want = k.kvpr_plan_split(prof, k.KVPR_COST_EQ10, 4, 64, 256, 2, 1)[0]
        splits, tim = k.kvpr_decode_step(st.ctx, 64, st.w, dev(st.x_in), st.x_out, None, timing=True)
        torch.cuda.synchronize()
        assert splits == [want] * 4
        assert all(t.split == want and t.ms_total > 0 for t in tim)
        base = st.x_out.cpu().numpy().copy()
        ref, _ = ko.decoder_stack_decode(st.layers, st.x_in, splits, st.stored)
        assert rel_err(base, ref) <= 5e-3
        for flags in (k.KVPR_DEBUG_SYNC, k.KVPR_DEBUG_POISON | k.KVPR_DEBUG_SYNC, k.KVPR_DEBUG_POISON):
            k.kvpr_set_debug(st.ctx, flags)
            k.kvpr_decode_step(st.ctx, 64, st.w, dev(st.x_in), st.x_out, None)
            torch.cuda.synchronize()
            assert np.array_equal(st.x_out.cpu().numpy(), base), flags
        k.kvpr_set_debug(st.ctx, 0)
    finally:
        st.close()


def test_decode_step_two_tokens(k):
    """Second token sees the rows the first token stored back in every layer."""
    n_layers, b, s, h, H, ffn = 3, 2, 24, 256, 2, 1024
    st = Stack(k, n_layers, b, s, h, H, ffn, max_seq=s + 4)
    try:
        splits = [5, 24, 0]
        k.kvpr_decode_step(st.ctx, s, st.w, dev(st.x_in), st.x_out, splits)
        torch.cuda.synchronize()
        _, trace = ko.decoder_stack_decode(st.layers, st.x_in, splits, st.stored)
        # oracle state after token 1: append xn to each layer's X; the stored cache is recomputed by the oracle
        layers2 = []
        for L, tr in zip(st.layers, trace):
            L2 = dict(L)
            L2["X"] = np.concatenate([np.asarray(L["X"], np.float64), tr["xn"][None]], 0)
            layers2.append(L2)
        x2 = kvpr_inputs._draw(np.random.default_rng(55), (b, h), 1.0)
        ref2, _ = ko.decoder_stack_decode(layers2, x2, [0, 0, 0])
        for splits2 in ([0, 0, 0], [25, 13, 1]):
            k.kvpr_decode_step(st.ctx, s + 1, st.w, dev(x2), st.x_out, splits2)
            torch.cuda.synchronize()
            assert rel_err(st.x_out.cpu().numpy(), ref2) <= 5e-3, splits2
    finally:
        st.close()


def test_six_steps_enqueued_without_waiting_equal_six_waited_for(k):
    """A caller that never synchronises between tokens (the library lets at most two steps of a context be in flight and
    blocks the caller for the rest) gets bit for bit what a caller that waits after every step gets."""
    n_layers, b, s, h, H, ffn = 3, 4, 40, 256, 2, 1024
    rng = np.random.default_rng(3)
    xs = [dev(kvpr_inputs._draw(rng, (b, h), 1.0)) for _ in range(6)]
    splits = [[int(v) for v in rng.integers(0, s + t + 1, n_layers)] for t in range(6)]
    outs = {}
    for mode in ("waited", "free"):
        st = Stack(k, n_layers, b, s, h, H, ffn, max_seq=s + 8)
        try:
            res = [torch.empty((b, h), dtype=torch.float16, device="cuda") for _ in range(6)]
            for t in range(6):
                k.kvpr_decode_step(st.ctx, s + t, st.w, xs[t], res[t], splits[t])
                if mode == "waited":
                    torch.cuda.synchronize()
            torch.cuda.synchronize()
            outs[mode] = [r.cpu().numpy() for r in res]
        finally:
            st.close()
    for t in range(6):
        assert np.isfinite(outs["free"][t].astype(np.float32)).all()
        assert np.array_equal(outs["free"][t], outs["waited"][t]), t


def test_decode_step_needs_ffn(k):
    ctx = k.kvpr_create(2, 256, 2, 128, 0, 2, 8)
    try:
        with pytest.raises(k.KvprError) as e:
            k.kvpr_decode_step(ctx, 4, [k.kvpr_layer_weights(), k.kvpr_layer_weights()], 1, 1, None)
        assert e.value.code == k.KVPR_E_STATE
    finally:
        k.kvpr_destroy(ctx)


def test_greedy_next_matches_oracle(k):
    b, h, vocab = 5, 256, 1000 + 7
    rng = np.random.default_rng(21)
    hidden = rng.standard_normal((b, h)).astype(np.float16)
    W_lm = (rng.standard_normal((h, vocab)) * 0.05).astype(np.float16)
    emb = rng.standard_normal((vocab, h)).astype(np.float16)
    logits = torch.empty((b, vocab), dtype=torch.float32, device="cuda")
    tokens = torch.empty((b,), dtype=torch.int32, device="cuda")
    x_next = torch.empty((b, h), dtype=torch.float16, device="cuda")
    k.kvpr_greedy_next(dev(hidden), dev(W_lm.T), dev(emb), b, h, vocab, logits, tokens, x_next)
    torch.cuda.synchronize()
    want_tok, want_logits, want_x = ko.greedy_next(hidden, W_lm, emb)
    got_logits = logits.cpu().numpy()
    assert rel_err(got_logits, want_logits) <= 1e-5
    got_tok = tokens.cpu().numpy()
    for n in range(b):
        # the argmax is unique unless the top two float64 logits are closer than the float32 error
        top2 = np.sort(want_logits[n])[-2:]
        if top2[1] - top2[0] > 1e-4 * abs(top2[1]):
            assert got_tok[n] == want_tok[n], n
        assert got_logits[n, got_tok[n]] == got_logits[n].max()
        assert np.array_equal(x_next.cpu().numpy()[n], emb[got_tok[n]])
    # ties go to the lowest index
    flat = torch.zeros((2, 128), dtype=torch.float16, device="cuda")
    wz = torch.zeros((300, 128), dtype=torch.float16, device="cuda")
    lg = torch.empty((2, 300), dtype=torch.float32, device="cuda")
    tk = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    k.kvpr_greedy_next(flat, wz, None, 2, 128, 300, lg, tk, None)
    torch.cuda.synchronize()
    assert tk.cpu().tolist() == [0, 0]


def test_full_depth_reduced_width(k):
    """The bench's stack depth (40 layers) at reduced width: errors must not build up through the residual stream."""
    n_layers, b, s, h, H, ffn = 40, 4, 256, 512, 4, 2048
    st = Stack(k, n_layers, b, s, h, H, ffn, seed0=700)
    try:
        rng = np.random.default_rng(3)
        splits = [int(v) for v in rng.integers(0, s + 1, n_layers)]
        splits[0], splits[1], splits[2] = 0, s, 192
        print("full depth, reduced width: 40 layers", flush=True)
        got_splits, _ = k.kvpr_decode_step(st.ctx, s, st.w, dev(st.x_in), st.x_out, splits)
        torch.cuda.synchronize()
        assert got_splits == splits
        ref, _ = ko.decoder_stack_decode(st.layers, st.x_in, splits, st.stored)
        got = st.x_out.cpu().numpy()
        assert np.isfinite(got).all()
        assert rel_err(got, ref) <= 1e-2
    finally:
        st.close()
