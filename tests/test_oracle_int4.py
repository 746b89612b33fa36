"""Pins for the 4-bit cache codec oracle: hand-worked groups, exactness where the arithmetic is
exact, the error bound of uniform quantisation, and the byte layout."""
import numpy as np
import pytest

from oracle import kvpr_int4_oracle as qo


def _row(vals):
    return np.asarray(vals, dtype=np.float16)[None]


def test_hand_group_integers():
    # values 0..15 four times: mn = 0, mx = 15, scale = 1 -> code = value, reconstruction exact
    v = np.tile(np.arange(16), 4)
    codes, scale, mn = qo.quantize_rows(_row(v))
    assert scale[0, 0] == 1.0 and mn[0, 0] == 0.0
    assert np.array_equal(codes[0], v)
    assert np.array_equal(qo.dequantize_rows(codes, scale, mn)[0], v.astype(np.float16))


def test_hand_group_shifted_and_scaled():
    # x = -3 + 0.5 k for k in 0..15 (exact in float16), padded with the minimum: mn = -3, mx = 4.5, scale = 0.5
    k = np.arange(64) % 16
    x = -3.0 + 0.5 * k
    codes, scale, mn = qo.quantize_rows(_row(x))
    assert scale[0, 0] == 0.5 and mn[0, 0] == -3.0
    assert np.array_equal(codes[0], k)
    assert np.array_equal(qo.roundtrip(_row(x))[0].astype(np.float64), x)


def test_rounding_is_half_to_even_and_clipped():
    # mn = 0, mx = 15 -> scale 1; 0.5 -> 0, 1.5 -> 2, 2.5 -> 2, 14.5 -> 14; nothing exceeds 15
    x = np.zeros(64)
    x[:6] = [0.0, 15.0, 0.5, 1.5, 2.5, 14.5]
    codes, _, _ = qo.quantize_rows(_row(x))
    assert codes[0, :6].tolist() == [0, 15, 0, 2, 2, 14]
    assert codes.max() == 15
    # the clip is live only for subnormal spans: span 22 ulps -> scale = fp16(22/15 ulp) = 1 ulp -> 22 steps -> 15
    tiny = np.zeros(64)
    tiny[1], tiny[2] = 22 * 2.0 ** -24, 7 * 2.0 ** -24
    codes, scale, mn = qo.quantize_rows(_row(tiny))
    assert scale[0, 0] == np.float16(2.0 ** -24) and codes[0, :3].tolist() == [0, 15, 7]
    assert qo.dequantize_rows(codes, scale, mn)[0, 1] == np.float16(15 * 2.0 ** -24)


def test_constant_group_and_extremes():
    x = np.full(64, 0.37, dtype=np.float16)
    codes, scale, mn = qo.quantize_rows(x[None])
    assert scale[0, 0] == 0 and not codes.any()
    assert np.array_equal(qo.roundtrip(x[None])[0], x)
    rng = np.random.default_rng(0)
    kv = rng.standard_normal((5, 3, 256)).astype(np.float16)
    codes, scale, mn = qo.quantize_rows(kv)
    rec = qo.dequantize_rows(codes, scale, mn)
    g = kv.reshape(5, 3, 4, 64)
    r = rec.reshape(5, 3, 4, 64)
    # the group minimum is reproduced exactly, every element within half a step (+ float16 rounding)
    assert np.array_equal(r.min(-1), g.min(-1))
    step = scale.astype(np.float64)[..., None]
    assert np.all(np.abs(r.astype(np.float64) - g.astype(np.float64)) <= 0.5 * step + 2e-3 * np.abs(g.astype(np.float64)) + 1e-3)
    assert codes.min() == 0 and codes.max() == 15


def test_pack_layout_and_roundtrip():
    h = 128
    rng = np.random.default_rng(1)
    kv = rng.standard_normal((4, 2, 2 * h)).astype(np.float16)
    codes, scale, mn = qo.quantize_rows(kv)
    packed = qo.pack_rows(codes, scale, mn)
    assert packed.shape == (4, 2, qo.packed_bytes(2 * h)) and qo.packed_bytes(2 * h) == 9 * h // 8 and qo.packed_bytes(h) == 9 * h // 16
    # element 2k in the low nibble of byte k, 2k+1 in the high nibble
    assert packed[1, 1, 7] == (codes[1, 1, 14] | (codes[1, 1, 15] << 4))
    # metadata follows the codes: (scale, mn) float16 pairs, group 0 first
    meta = packed[1, 1, h:h + 4].copy().view(np.float16)
    assert meta[0] == scale[1, 1, 0] and meta[1] == mn[1, 1, 0]
    c2, s2, m2 = qo.unpack_rows(packed, 2 * h)
    assert np.array_equal(c2, codes) and np.array_equal(s2, scale) and np.array_equal(m2, mn)
    assert qo.packed_bytes(2 * 4096) * 32 * 1024 == 150_994_944   # 9h/8 * b * s, against 536 870 912 B in float16


def test_layer_decode_over_compressed_store():
    import kvpr_inputs
    from oracle import kvpr_oracle as ko

    lay = kvpr_inputs.make_layer(5, 2, 24, 128, 2)
    exact = ko.layer_decode(lay, 0)["o"]
    # everything recomputed from uncompressed activations: the codec is never touched
    assert np.array_equal(qo.layer_decode_int4(lay, 24, compress_x=False)["o"], ko.layer_decode(lay, 24)["o"])
    # the new token's row is exact at every split, the transferred rows are the round trip of the stored ones
    r = qo.layer_decode_int4(lay, 8)
    st = ko.stored_kv(lay)
    assert np.array_equal(r["kv"][24], ko.layer_decode(lay, 8)["kv"][24])
    assert np.array_equal(r["kv"][8:24], qo.roundtrip(st[8:24].astype(np.float16)).astype(np.float64))
    assert not np.array_equal(r["kv"][:8], st[:8])           # recomputed from compressed activations
    for l in (0, 8, 24):
        o = qo.layer_decode_int4(lay, l)["o"]
        err = np.abs(o - exact).max() / np.abs(exact).max()
        assert 0 < err < 0.08, (l, err)                       # lossy, but a 4-bit-sized perturbation
