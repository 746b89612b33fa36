"""Pins for oracle/kvpr_oracle.py against things other than itself: a hand-worked
example, closed forms, textbook special cases through torch CPU routines, and a
second scalar-loop implementation with exactly rounded sums."""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import kvpr_inputs
from oracle import kvpr_oracle as ko


def _tiny(seed=0, b=2, s=5, h=8, H=2):
    return kvpr_inputs.make_layer(seed, b, s, h, H, w_scale=0.3, b_scale=0.1)


def _load_hand(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "hand_example.json")))
    c = math.sqrt(2.0) * math.log(2.0)
    layer = {k: np.array(g[k], dtype=np.float64) for k in ("X", "x_new", "Wq", "Wv", "Wo", "bq", "bk", "bv", "bo")}
    layer["Wk"] = c * np.eye(4)
    layer["n_heads"] = g["n_heads"]
    return g, layer


# ---- P4: hand-worked example (Eq. 1,2,3,5,7) --------------------------------
@pytest.mark.parametrize("l", [0, 1, 2])
def test_hand_example(golden_dir, l):
    g, layer = _load_hand(golden_dir)
    stored = ko.stored_kv(layer, kv_round="none")
    np.testing.assert_allclose(stored[:, 0, 4:], np.array(g["expect_V_rows"][:2]), rtol=0, atol=1e-15)
    r = ko.layer_decode(layer, l, kv_stored=stored, kv_round="none")
    np.testing.assert_allclose(r["kv"][:, 0, 4:], np.array(g["expect_V_rows"]), rtol=0, atol=1e-15)
    z = np.array([float(Fraction(v)) for v in g["expect_z"]])
    o = np.array([float(Fraction(v)) for v in g["expect_o"]])
    np.testing.assert_allclose(r["z"][0], z, rtol=1e-14)
    np.testing.assert_allclose(r["o"][0], o, rtol=1e-14)
    rl = ko.layer_decode_loops(layer, l, kv_stored=stored)
    np.testing.assert_allclose(rl["o"][0], o, rtol=1e-14)


def test_hand_example_probabilities(golden_dir):
    """The softmax weights themselves: uniform V picks them out of z."""
    g, layer = _load_hand(golden_dir)
    # V_j = e_j-like: make V rows the indicator of position j in both heads' first column
    S = 3
    q = ko.project(layer["x_new"], layer["Wq"], layer["bq"])
    kv = ko.assemble_kv(2, layer["X"], ko.stored_kv(layer, "none"), layer["x_new"], layer["Wk"], layer["Wv"],
                        layer["bk"], layer["bv"], kv_round="none")
    for j in range(S):
        kvj = kv.copy()
        kvj[:, :, 4:] = 0.0
        kvj[j, :, 4:] = 1.0
        z = ko.decode_attention(q, kvj, 2)[0]
        assert z[0] == pytest.approx(float(Fraction(g["expect_p_head0"][j])), rel=1e-14)
        assert z[2] == pytest.approx(float(Fraction(g["expect_p_head1"][j])), rel=1e-14)


# ---- P1: recomputed rows equal stored rows (Eq. 7 is Eq. 1 on rows [0,l)) ----
def test_recompute_equals_stored():
    layer = _tiny(1, b=3, s=9, h=16, H=4)
    stored = ko.stored_kv(layer, "fp16")
    for l in range(10):
        rec = ko.round_fp16(ko.recompute_kv(layer["X"][:l], layer["Wk"], layer["Wv"], layer["bk"], layer["bv"]))
        assert np.array_equal(rec, stored[:l])
    full = ko.stored_kv(layer, "none")
    rec = ko.recompute_kv(layer["X"][:4], layer["Wk"], layer["Wv"], layer["bk"], layer["bv"])
    np.testing.assert_allclose(rec, full[:4], rtol=1e-13, atol=1e-15)


# ---- P2: the output does not depend on the split ----------------------------
def test_split_invariance_bit_exact():
    layer = _tiny(2, b=2, s=12, h=16, H=2)
    stored = ko.stored_kv(layer, "fp16")
    ref = ko.layer_decode(layer, 0, stored)
    for l in range(1, 13):
        r = ko.layer_decode(layer, l, stored)
        assert np.array_equal(r["kv"], ref["kv"])
        assert np.array_equal(r["o"], ref["o"])


def test_split_invariance_exact_sums():
    layer = _tiny(3, b=1, s=4, h=8, H=2)
    ref = ko.layer_decode_loops(layer, 0)
    for l in range(1, 5):
        assert np.array_equal(ko.layer_decode_loops(layer, l)["o"], ref["o"])


def test_wrong_stored_cache_is_visible():
    """The transferred rows really are used: corrupt row l..s and the output moves; rows < l are ignored."""
    layer = _tiny(4, b=2, s=6, h=8, H=2)
    stored = ko.stored_kv(layer, "fp16")
    bad = stored.copy()
    bad[1] += 1.0
    ref = ko.layer_decode(layer, 0, stored)["o"]
    assert np.array_equal(ko.layer_decode(layer, 2, bad)["o"], ref)       # row 1 recomputed
    assert not np.allclose(ko.layer_decode(layer, 1, bad)["o"], ref)      # row 1 transferred


# ---- numpy version against the scalar-loop version --------------------------
@pytest.mark.parametrize("seed,b,s,h,H", [(5, 2, 5, 8, 2), (6, 1, 3, 12, 3), (7, 3, 2, 4, 1)])
def test_vectorised_matches_loops(seed, b, s, h, H):
    layer = _tiny(seed, b, s, h, H)
    for l in (0, s // 2, s):
        a = ko.layer_decode(layer, l, kv_round="none")
        c = ko.layer_decode_loops(layer, l)
        np.testing.assert_allclose(a["kv"], c["kv"], rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(a["z"], c["z"], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(a["o"], c["o"], rtol=1e-12, atol=1e-15)


# ---- P3: textbook special cases through torch CPU ---------------------------
def _torch_reference(layer):
    """Last row of causal self-attention over the s+1 inputs, with nn.functional routines (float64)."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    X = torch.cat([t(layer["X"]), t(layer["x_new"])[None]], 0)             # [s+1, b, h]
    b, h, H = X.shape[1], X.shape[2], layer["n_heads"]
    d = h // H
    lin = lambda x, W, bias: torch.nn.functional.linear(x, t(W).T.contiguous(), t(bias))
    Q, K, V = (lin(X, layer[w], layer[bb]) for w, bb in (("Wq", "bq"), ("Wk", "bk"), ("Wv", "bv")))
    to_heads = lambda a: a.permute(1, 0, 2).reshape(b, -1, H, d).permute(0, 2, 1, 3)   # [b,H,S,d]
    Z = torch.nn.functional.scaled_dot_product_attention(to_heads(Q), to_heads(K), to_heads(V), is_causal=True)
    z_last = Z[:, :, -1, :].reshape(b, h)
    return lin(z_last, layer["Wo"], layer["bo"]).numpy(), z_last.numpy()


@pytest.mark.parametrize("seed,b,s,h,H", [(8, 2, 17, 32, 4), (9, 3, 8, 64, 1), (10, 1, 33, 24, 3)])
def test_full_recompute_is_causal_attention_last_row(seed, b, s, h, H):
    layer = _tiny(seed, b, s, h, H)
    o_ref, z_ref = _torch_reference(layer)
    for l in (0, s // 3, s):
        r = ko.layer_decode(layer, l, kv_round="none")
        np.testing.assert_allclose(r["z"], z_ref, rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(r["o"], o_ref, rtol=1e-11, atol=1e-13)


def test_fp16_cache_mode_is_close_to_unrounded():
    layer = kvpr_inputs.make_layer(11, 2, 20, 64, 4)
    a = ko.layer_decode(layer, 7, kv_round="none")["o"]
    c = ko.layer_decode(layer, 7, kv_round="fp16")["o"]
    assert np.max(np.abs(a - c)) <= 2e-3 * np.max(np.abs(a))
    assert not np.array_equal(a, c)


# ---- P5: softmax invariants --------------------------------------------------
def test_key_bias_does_not_change_output():
    """Adding bk shifts every score of a head by the same q.bk, which softmax cancels."""
    layer = _tiny(12, b=2, s=7, h=16, H=4)
    a = ko.layer_decode(layer, 3, kv_round="none")["o"]
    layer2 = dict(layer)
    layer2["bk"] = np.linspace(-2, 3, 16)
    c = ko.layer_decode(layer2, 3, kv_round="none")["o"]
    np.testing.assert_allclose(a, c, rtol=1e-11, atol=1e-13)


def test_equal_keys_average_the_values():
    rng = np.random.default_rng(13)
    b, h, H, S = 2, 12, 3, 9
    kv = rng.standard_normal((S, b, 2 * h))
    kv[:, :, :h] = kv[0:1, :, :h]                       # same key at every position
    q = rng.standard_normal((b, h))
    z = ko.decode_attention(q, kv, H)
    np.testing.assert_allclose(z, kv[:, :, h:].mean(axis=0), rtol=1e-12)


def test_one_dominant_key_selects_its_value():
    b, h, H, S = 1, 8, 2, 5
    kv = np.zeros((S, b, 2 * h))
    kv[:, :, h:] = np.arange(S)[:, None, None] + np.arange(h)[None, None, :] * 10.0
    kv[3, 0, :4] = 200.0        # head 0 prefers position 3
    kv[1, 0, 4:8] = 200.0       # head 1 prefers position 1
    z = ko.decode_attention(np.ones((b, h)), kv, H)[0]
    np.testing.assert_allclose(z[:4], kv[3, 0, h:h + 4], rtol=1e-12)
    np.testing.assert_allclose(z[4:], kv[1, 0, h + 4:], rtol=1e-12)


def test_scale_is_inverse_sqrt_head_dim():
    """Two positions, one head of d=4: p1/p0 = exp((q.k1 - q.k0)/2)."""
    kv = np.zeros((2, 1, 8))
    kv[1, 0, :4] = [1.0, 0.0, 0.0, 0.0]
    kv[0, 0, 4:] = [1, 0, 0, 0]
    kv[1, 0, 4:] = [0, 1, 0, 0]
    q = np.array([[3.0, 0, 0, 0]])
    z = ko.decode_attention(q, kv, 1)[0]
    assert z[1] / z[0] == pytest.approx(math.exp(3.0 / 2.0), rel=1e-13)


# ---- rest of the decoder layer -----------------------------------------------
def test_layer_norm_and_ffn_match_torch():
    rng = np.random.default_rng(14)
    x = rng.standard_normal((3, 16))
    g, beta = rng.standard_normal(16), rng.standard_normal(16)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    ref = torch.nn.functional.layer_norm(t(x), (16,), t(g), t(beta), 1e-5).numpy()
    np.testing.assert_allclose(ko.layer_norm(x, g, beta), ref, rtol=1e-12, atol=1e-14)
    W1, W2 = rng.standard_normal((16, 40)), rng.standard_normal((40, 16))
    b1, b2 = rng.standard_normal(40), rng.standard_normal(16)
    ref = torch.nn.functional.linear(torch.relu(torch.nn.functional.linear(t(x), t(W1).T, t(b1))), t(W2).T, t(b2)).numpy()
    np.testing.assert_allclose(ko.ffn(x, W1, b1, W2, b2), ref, rtol=1e-12, atol=1e-13)
