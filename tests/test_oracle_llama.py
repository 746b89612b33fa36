"""Pins for the LLaMA-shaped oracle: the rotary embedding against its complex-number definition and its
defining properties, RMSNorm / SiLU closed forms, and split invariance of the rotary layer."""
import numpy as np
import pytest

import kvpr_inputs
from oracle import kvpr_llama_oracle as lo
from oracle import kvpr_oracle as ko


def test_rope_hand_values():
    # one head of width 2: theta_0 = 1, so position p rotates the pair (x0, x1) by p radians
    x = np.array([[3.0, 4.0]])
    y = lo.rope(x, [np.pi / 2], 1)
    assert np.allclose(y, [[-4.0, 3.0]], atol=1e-15)
    y = lo.rope(x, [np.pi], 1)
    assert np.allclose(y, [[-3.0, -4.0]], atol=1e-15)
    # width 4: pairs are (0, 2) and (1, 3); theta = [1, 10000^(-1/2)] = [1, 0.01]
    x = np.array([[1.0, 2.0, 0.0, 0.0]])
    p = 7.0
    want = [np.cos(p), 2 * np.cos(0.01 * p), np.sin(p), 2 * np.sin(0.01 * p)]
    assert np.allclose(lo.rope(x, [p], 1), [want], atol=1e-15)
    assert np.allclose(lo.rope_angles([3], 8)[0], [3.0, 3 * 10 ** -1.0, 3 * 10 ** -2.0, 3 * 10 ** -3.0], rtol=1e-14)


def test_rope_is_the_complex_rotation_per_pair():
    rng = np.random.default_rng(0)
    H, d, P = 3, 16, 11
    x = rng.standard_normal((P, 2, H * d))
    pos = rng.integers(0, 5000, P)
    y = lo.rope(x, pos, H)
    xh = x.reshape(P, 2, H, d)
    z = xh[..., : d // 2] + 1j * xh[..., d // 2:]
    theta = 10000.0 ** (-2.0 * np.arange(d // 2) / d)
    w = z * np.exp(1j * pos[:, None, None, None] * theta)
    want = np.concatenate([w.real, w.imag], -1).reshape(P, 2, H * d)
    assert np.allclose(y, want, rtol=1e-12, atol=1e-12)


def test_rope_properties():
    rng = np.random.default_rng(1)
    H, d = 2, 8
    q = rng.standard_normal((1, H * d))
    k = rng.standard_normal((1, H * d))
    # position 0 is the identity; norms per head are preserved
    assert np.array_equal(lo.rope(q, [0], H), q)
    y = lo.rope(q, [123], H)
    assert np.allclose(np.linalg.norm(y.reshape(H, d), axis=1), np.linalg.norm(q.reshape(H, d), axis=1), rtol=1e-13)
    # scores depend on the position difference only
    def score(m, n):
        a = lo.rope(q, [m], H).reshape(H, d)
        b = lo.rope(k, [n], H).reshape(H, d)
        return (a * b).sum(-1)
    assert np.allclose(score(10, 3), score(107, 100), rtol=1e-11)
    assert not np.allclose(score(10, 3), score(10, 4))
    # rotations compose: position m then n equals m + n
    assert np.allclose(lo.rope(lo.rope(q, [5], H), [9], H), lo.rope(q, [14], H), rtol=1e-12, atol=1e-13)


def test_norm_and_activation_closed_forms():
    x = np.full((2, 16), 3.0)
    g = np.linspace(0.5, 2.0, 16)
    assert np.allclose(lo.rms_norm(x, g, eps=0.0), np.broadcast_to(g, (2, 16)), rtol=1e-15)
    y = np.random.default_rng(2).standard_normal((3, 32))
    assert np.allclose(lo.rms_norm(7.0 * y, np.ones(32), eps=0.0), lo.rms_norm(y, np.ones(32), eps=0.0), rtol=1e-13)
    assert np.allclose((lo.rms_norm(y, np.ones(32), eps=0.0) ** 2).mean(-1), 1.0, rtol=1e-13)
    assert lo.silu(0.0) == 0.0
    assert np.isclose(lo.silu(1.0), 1.0 / (1.0 + np.exp(-1.0)))
    assert np.isclose(lo.silu(-30.0), -30.0 * np.exp(-30.0), rtol=1e-9) and np.isclose(lo.silu(30.0), 30.0, rtol=1e-12)
    # gated FFN with identity-like matrices: down(silu(x) * x)
    eye = np.eye(4)
    v = np.array([[0.5, -1.0, 2.0, 0.0]])
    assert np.allclose(lo.gated_ffn(v, eye, eye, eye), lo.silu(v) * v)


def test_rotary_layer_is_split_invariant_and_position_aware():
    lay = kvpr_inputs.make_layer(3, 2, 20, 128, 2)
    st = lo.stored_kv(lay, "none")
    outs = [lo.layer_decode(lay, l, st, "none")["o"] for l in (0, 1, 7, 20)]
    for o in outs[1:]:
        assert np.allclose(o, outs[0], rtol=1e-11, atol=1e-13)       # recomputed rows equal the stored rows
    # the value half is not rotated, the key half is: V equals the OPT-shaped oracle's bias-free V, K does not
    plain = ko.recompute_kv(lay["X"], lay["Wk"], lay["Wv"])
    assert np.array_equal(st[..., 128:], plain[..., 128:])
    assert np.array_equal(st[0, :, :128], plain[0, :, :128]) and not np.allclose(st[5, :, :128], plain[5, :, :128])
    # scores computed from rotated q, k equal the scores of unrotated q, k rotated by the relative distance
    r = lo.layer_decode(lay, 0, st, "none")
    q_plain = ko.project(lay["x_new"], lay["Wq"])
    t = 13
    rel = lo.rope(q_plain[None], [20 - t], 2)[0]                       # q moved by (s - t), k left at 0
    a = (r["q"].reshape(2, 2, 64) * st[t, :, :128].reshape(2, 2, 64)).sum(-1)
    b = (rel.reshape(2, 2, 64) * plain[t, :, :128].reshape(2, 2, 64)).sum(-1)
    assert np.allclose(a, b, rtol=1e-10, atol=1e-12)
    # a wrong position for the new token changes the result
    lay2 = dict(lay, X=lay["X"][:19])
    assert not np.allclose(lo.layer_decode(lay2, 0, st[:19], "none")["o"], outs[0])


def test_stack_reduces_to_single_layer_pieces():
    h, H, ffn = 128, 2, 256
    L = kvpr_inputs.make_layer(9, 2, 12, h, H)
    L.update(kvpr_inputs.make_gated_ffn(9, h, ffn))
    x = kvpr_inputs._draw(np.random.default_rng(8), (2, h), 1.0)
    out, trace = lo.decoder_stack_decode([L], x, [5], None, "none", "none")
    xn = lo.rms_norm(x, L["ln1_g"])
    mid = x.astype(np.float64) + lo.layer_decode(dict(L, x_new=xn), 5, None, "none")["o"]
    want = mid + lo.gated_ffn(lo.rms_norm(mid, L["ln2_g"]), L["Wg"], L["Wu"], L["Wd"])
    assert np.allclose(out, want, rtol=1e-12, atol=1e-13)
    assert np.allclose(trace[0]["xn"], xn)
