"""The pins must notice plausible mistakes: each mutation below plants one in a copy of the
oracle's source (never in the product) and the pin suite has to fail on it."""
import importlib.util
import json
import math
import os
import sys
import types
from fractions import Fraction

import numpy as np
import pytest
import torch

import kvpr_inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def _load(path, replace=None):
    src = open(path).read()
    if replace:
        old, new = replace
        assert src.count(old) >= 1, f"mutation target not found: {old!r}"
        src = src.replace(old, new, 1)
    mod = types.ModuleType("mutant_" + os.path.basename(path)[:-3])
    exec(compile(src, path, "exec"), mod.__dict__)
    return mod


# ---- compact pin suites (same facts as test_oracle_attention / test_oracle_plan) ----
def attention_pins_hold(ko) -> bool:
    try:
        g = json.load(open(os.path.join(GOLDEN, "hand_example.json")))
        layer = {k: np.array(g[k], dtype=np.float64) for k in ("X", "x_new", "Wq", "Wv", "Wo", "bq", "bk", "bv", "bo")}
        layer["Wk"] = math.sqrt(2.0) * math.log(2.0) * np.eye(4)
        layer["n_heads"] = 2
        o = np.array([float(Fraction(v)) for v in g["expect_o"]])
        for l in (0, 1, 2):
            r = ko.layer_decode(layer, l, kv_round="none")
            if not np.allclose(r["o"][0], o, rtol=1e-12):
                return False
        # textbook: last row of causal attention through torch, random asymmetric weights
        L = kvpr_inputs.make_layer(8, 2, 9, 16, 2, w_scale=0.3, b_scale=0.1)
        t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
        X = torch.cat([t(L["X"]), t(L["x_new"])[None]], 0)
        lin = lambda x, W, bias: torch.nn.functional.linear(x, t(W).T.contiguous(), t(bias))
        Q, K, V = (lin(X, L[w], L[bb]) for w, bb in (("Wq", "bq"), ("Wk", "bk"), ("Wv", "bv")))
        heads = lambda a: a.permute(1, 0, 2).reshape(2, -1, 2, 8).permute(0, 2, 1, 3)
        Z = torch.nn.functional.scaled_dot_product_attention(heads(Q), heads(K), heads(V), is_causal=True)
        ref = lin(Z[:, :, -1, :].reshape(2, 16), L["Wo"], L["bo"]).numpy()
        stored = ko.stored_kv(L, "none")
        outs = [ko.layer_decode(L, l, stored, kv_round="none")["o"] for l in (0, 4, 9)]
        if not all(np.allclose(o, ref, rtol=1e-10, atol=1e-12) for o in outs):
            return False
        # transferred rows are really used / recomputed rows really ignore the stored ones
        bad = stored.copy()
        bad[1] += 1.0
        if not np.allclose(ko.layer_decode(L, 2, bad, kv_round="none")["o"], ref, rtol=1e-10, atol=1e-12):
            return False
        if np.allclose(ko.layer_decode(L, 1, bad, kv_round="none")["o"], ref, rtol=1e-6):
            return False
        # fp16 cache mode: recomputed rows equal stored rows bit for bit
        st16 = ko.stored_kv(L, "fp16")
        if not np.array_equal(ko.assemble_kv(5, L["X"], st16, L["x_new"], L["Wk"], L["Wv"], L["bk"], L["bv"])[:9], st16):
            return False
        return True
    except Exception:
        return False


def plan_pins_hold(po) -> bool:
    try:
        toy = dict(b=1, s=9, h=1, p=1, v_com=1.0, v_gpu=4.0)
        if [po.cost(po.COST_EQ10, l, **toy) for l in range(10)] != [18, 17, 16, 15, 14, 13, 12, 14, 16, 18]:
            return False
        if [po.cost(po.COST_ROW, l, **toy) for l in range(10)] != [18, 16, 14, 12, 10, 8, 6, 7, 8, 9]:
            return False
        if po.plan_split(po.COST_NS, **toy) != (4, 10.0):
            return False
        t1 = json.load(open(os.path.join(GOLDEN, "table1_kv_sizes.json")))
        for row in t1["rows"]:
            if po.bytes_kv(32, 0, 1024, row["hidden"], 2) != row["kv_MB"] * 2 ** 20:
                return False
        if po.flops_recompute(32, 1024, 4096) != 2199023255552:
            return False
        fig = json.load(open(os.path.join(GOLDEN, "fig_split_points.json")))
        fit = json.load(open(os.path.join(GOLDEN, "fig_split_ratio.json")))
        v_com = fit["v_com_bytes_per_s"]
        got = [po.plan_split(po.COST_EQ10, 64, 256 + i, 4096, 2, v_com, fit["ratio_flop_per_byte_mid"] * v_com)[0]
               for i in fig["tokens_generated"]]
        return got == fig["split_l"]
    except Exception:
        return False


ORACLE = os.path.join(ROOT, "oracle", "kvpr_oracle.py")
PLAN = os.path.join(ROOT, "oracle", "kvpr_plan_oracle.py")


def test_unmutated_sources_pass():
    assert attention_pins_hold(_load(ORACLE))
    assert plan_pins_hold(_load(PLAN))


ATTENTION_MUTATIONS = [
    ("scale by d instead of sqrt(d)", ("/ math.sqrt(d)\n    scores = scores - scores.max", "/ d\n    scores = scores - scores.max")),
    ("transposed weight", ("y = _f64(x) @ _f64(W)", "y = _f64(x) @ _f64(W).T")),
    ("bias dropped", ("        y = y + _f64(bias)", "        y = y + 0.0 * _f64(bias)")),
    ("K and V halves swapped", ("return np.concatenate([K, V], axis=-1)", "return np.concatenate([V, K], axis=-1)")),
    ("transferred rows taken one position early", ("             _f64(kv_stored)[l:s],", "             _f64(kv_stored)[max(l - 1, 0):s][:s - l],")),
    ("new token's row left out of the softmax", ('    z = np.einsum("bij,jbid->bid", p, V)', '    p[:, :, -1] = 0.0\n    z = np.einsum("bij,jbid->bid", p, V)')),
    ("heads interleaved instead of contiguous", ("qh = q.reshape(b, n_heads, d)", "qh = q.reshape(b, d, n_heads).transpose(0, 2, 1)")),
    ("output projection skipped bias", ('    o = project(z, layer["Wo"], layer["bo"])', '    o = project(z, layer["Wo"])')),
    ("query uses key weights", ('    q = project(layer["x_new"], layer["Wq"], layer["bq"])', '    q = project(layer["x_new"], layer["Wk"], layer["bq"])')),
    ("softmax not normalised", ("    p = p / p.sum(axis=-1, keepdims=True)", "    p = p / 1.0")),
]


@pytest.mark.parametrize("name,replace", ATTENTION_MUTATIONS, ids=[m[0] for m in ATTENTION_MUTATIONS])
def test_attention_pins_catch(name, replace):
    assert not attention_pins_hold(_load(ORACLE, replace)), name


PLAN_MUTATIONS = [
    ("first term of Eq. 10 dropped", ("return t_act + max(t_rc, t_kv)", "return max(t_rc, t_kv)")),
    ("cache bytes without the factor 2", ("return 2 * b * (s - l) * h * p", "return b * (s - l) * h * p")),
    ("flops 2bh^2 per position", ("return 4 * b * l * h * h", "return 2 * b * l * h * h")),
    ("max replaced by sum", ("return t_act + max(t_rc, t_kv)", "return t_act + t_rc + t_kv")),
    ("ties to the largest l", ("        if t < best_t:\n            best_l, best_t = l, t\n    return best_l, best_t\n\n\n#", "        if t <= best_t:\n            best_l, best_t = l, t\n    return best_l, best_t\n\n\n#")),
    ("activation bytes off by one position", ("return b * l * h * p", "return b * (l + 1) * h * p")),
    ("row form keeps the first term", ("        return max(t_rc, t_kv)\n    if model == COST_NS", "        return t_act + max(t_rc, t_kv)\n    if model == COST_NS")),
]


@pytest.mark.parametrize("name,replace", PLAN_MUTATIONS, ids=[m[0] for m in PLAN_MUTATIONS])
def test_plan_pins_catch(name, replace):
    assert not plan_pins_hold(_load(PLAN, replace)), name


# ---- 4-bit store codec (Sec. 4.4) ----
def int4_pins_hold(qo) -> bool:
    try:
        row = lambda v: np.asarray(v, dtype=np.float16)[None]
        v = np.tile(np.arange(16), 4)
        codes, scale, mn = qo.quantize_rows(row(v))
        if scale[0, 0] != 1.0 or mn[0, 0] != 0.0 or not np.array_equal(codes[0], v):
            return False
        if not np.array_equal(qo.dequantize_rows(codes, scale, mn)[0], v.astype(np.float16)):
            return False
        kk = np.arange(64) % 16
        x = -3.0 + 0.5 * kk
        codes, scale, mn = qo.quantize_rows(row(x))
        if scale[0, 0] != 0.5 or mn[0, 0] != -3.0 or not np.array_equal(codes[0], kk):
            return False
        if not np.array_equal(qo.roundtrip(row(x))[0].astype(np.float64), x):
            return False
        y = np.zeros(64)
        y[:6] = [0.0, 15.0, 0.5, 1.5, 2.5, 14.5]
        if qo.quantize_rows(row(y))[0][0, :6].tolist() != [0, 15, 0, 2, 2, 14]:
            return False
        c = np.full(64, 0.37, dtype=np.float16)
        if not np.array_equal(qo.roundtrip(c[None])[0], c):
            return False
        tiny = np.zeros(64)
        tiny[1] = 22 * 2.0 ** -24                       # subnormal span: the scale rounds down to one ulp, 22 steps fit
        if qo.quantize_rows(row(tiny))[0][0, :2].tolist() != [0, 15]:
            return False
        rng = np.random.default_rng(0)
        kv = rng.standard_normal((5, 3, 256)).astype(np.float16)
        codes, scale, mn = qo.quantize_rows(kv)
        rec = qo.dequantize_rows(codes, scale, mn)
        g, r = kv.reshape(5, 3, 4, 64).astype(np.float64), rec.reshape(5, 3, 4, 64).astype(np.float64)
        if not np.array_equal(r.min(-1), g.min(-1)) or codes.max() != 15 or codes.min() != 0:
            return False
        if not np.all(np.abs(r - g) <= 0.5 * scale.astype(np.float64)[..., None] + 2e-3 * np.abs(g) + 1e-3):
            return False
        packed = qo.pack_rows(codes, scale, mn)
        if packed.shape != (5, 3, 144) or qo.packed_bytes(256) != 144:
            return False
        if packed[1, 1, 7] != (codes[1, 1, 14] | (codes[1, 1, 15] << 4)):
            return False
        meta = packed[1, 1, 128:132].copy().view(np.float16)
        if meta[0] != scale[1, 1, 0] or meta[1] != mn[1, 1, 0]:
            return False
        c2, s2, m2 = qo.unpack_rows(packed, 256)
        return np.array_equal(c2, codes) and np.array_equal(s2, scale) and np.array_equal(m2, mn)
    except Exception:
        return False


INT4 = os.path.join(ROOT, "oracle", "kvpr_int4_oracle.py")
INT4_MUTATIONS = [
    ("16 levels spread over 16 steps", ("(mx - mn) / np.float32(15.0)", "(mx - mn) / np.float32(16.0)")),
    ("truncation instead of rounding", ("q = np.rint((g - mn[..., None]) / safe[..., None])", "q = np.floor((g - mn[..., None]) / safe[..., None])")),
    ("offset from the maximum", ("q = np.rint((g - mn[..., None]) / safe[..., None])", "q = np.rint((g - mx[..., None]) / safe[..., None])")),
    ("codes clipped to 16", ("codes = np.clip(q, 0, 15)", "codes = np.clip(q, 0, 16)")),
    ("groups of 32", ("GROUP = 64", "GROUP = 32")),
    ("nibbles swapped", ("nib = (lo | (hi << 4))", "nib = (hi | (lo << 4))")),
    ("minimum dropped on the way back", ("x = (prod + mn16.astype(np.float32)[..., None])", "x = (prod + 0 * mn16.astype(np.float32)[..., None])")),
    ("metadata order swapped", ("meta = np.stack([scale16, mn16], axis=-1)", "meta = np.stack([mn16, scale16], axis=-1)")),
    ("scale kept in float32", ("scale16 = ((mx - mn) / np.float32(15.0)).astype(np.float16)\n", "scale16 = ((mx - mn) / np.float32(15.0))\n")),
]


def test_int4_unmutated_passes():
    assert int4_pins_hold(_load(INT4))


@pytest.mark.parametrize("name,replace", INT4_MUTATIONS, ids=[m[0] for m in INT4_MUTATIONS])
def test_int4_pins_catch(name, replace):
    assert not int4_pins_hold(_load(INT4, replace)), name


# ---- rotary / LLaMA-shaped layer ----
def llama_pins_hold(lo) -> bool:
    try:
        from oracle import kvpr_oracle as ko
        x = np.array([[3.0, 4.0]])
        if not np.allclose(lo.rope(x, [np.pi / 2], 1), [[-4.0, 3.0]], atol=1e-15):
            return False
        x4 = np.array([[1.0, 2.0, 0.0, 0.0]])
        p = 7.0
        if not np.allclose(lo.rope(x4, [p], 1), [[np.cos(p), 2 * np.cos(0.01 * p), np.sin(p), 2 * np.sin(0.01 * p)]], atol=1e-15):
            return False
        rng = np.random.default_rng(1)
        H, d = 2, 8
        q, kx = rng.standard_normal((1, H * d)), rng.standard_normal((1, H * d))
        sc = lambda m, n: (lo.rope(q, [m], H).reshape(H, d) * lo.rope(kx, [n], H).reshape(H, d)).sum(-1)
        if not np.allclose(sc(10, 3), sc(107, 100), rtol=1e-11) or not np.array_equal(lo.rope(q, [0], H), q):
            return False
        lay = kvpr_inputs.make_layer(3, 2, 20, 128, 2)
        st = lo.stored_kv(lay, "none")
        outs = [lo.layer_decode(lay, l, st, "none")["o"] for l in (0, 7, 20)]
        if not all(np.allclose(o, outs[0], rtol=1e-11, atol=1e-13) for o in outs):
            return False
        plain = ko.recompute_kv(lay["X"], lay["Wk"], lay["Wv"])
        if not np.array_equal(st[..., 128:], plain[..., 128:]) or not np.array_equal(st[0, :, :128], plain[0, :, :128]):
            return False
        r = lo.layer_decode(lay, 0, st, "none")
        t = 13
        rel = lo.rope(ko.project(lay["x_new"], lay["Wq"])[None], [20 - t], 2)[0]
        a = (r["q"].reshape(2, 2, 64) * st[t, :, :128].reshape(2, 2, 64)).sum(-1)
        b = (rel.reshape(2, 2, 64) * plain[t, :, :128].reshape(2, 2, 64)).sum(-1)
        if not np.allclose(a, b, rtol=1e-10, atol=1e-12):
            return False
        # the new token's own key: its score with itself is the unrotated q . k
        k_new = ko.project(lay["x_new"], lay["Wk"])
        q_plain = ko.project(lay["x_new"], lay["Wq"])
        own = (r["q"].reshape(2, 2, 64) * r["kv"][20, :, :128].reshape(2, 2, 64)).sum(-1)
        if not np.allclose(own, (q_plain.reshape(2, 2, 64) * k_new.reshape(2, 2, 64)).sum(-1), rtol=1e-10, atol=1e-12):
            return False
        xc = np.full((2, 16), 3.0)
        gg = np.linspace(0.5, 2.0, 16)
        if not np.allclose(lo.rms_norm(xc, gg, eps=0.0), np.broadcast_to(gg, (2, 16)), rtol=1e-15):
            return False
        if not np.isclose(lo.silu(1.0), 1.0 / (1.0 + np.exp(-1.0))) or lo.silu(0.0) != 0.0:
            return False
        eye = np.eye(4)
        v = np.array([[0.5, -1.0, 2.0, 0.0]])
        return bool(np.allclose(lo.gated_ffn(v, eye, 2 * eye, eye), lo.silu(v) * 2 * v))
    except Exception:
        return False


LLAMA = os.path.join(ROOT, "oracle", "kvpr_llama_oracle.py")
LLAMA_MUTATIONS = [
    ("rotation backwards", ("out = np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)", "out = np.concatenate([x1 * c + x2 * s, x2 * c - x1 * s], axis=-1)")),
    ("adjacent pairs instead of half split", ("x1, x2 = xh[..., : d // 2], xh[..., d // 2:]", "x1, x2 = xh[..., 0::2], xh[..., 1::2]")),
    ("angle exponent i/d", ("theta = base ** (-2.0 * i / d)", "theta = base ** (-1.0 * i / d)")),
    ("recomputed rows one position late", ("np.arange(pos0, pos0 + l), n_heads, base)", "np.arange(pos0 + 1, pos0 + l + 1), n_heads, base)")),
    ("new token rotated with position s - 1", ('    q = rope(project(x_new, layer["Wq"])[None], [s], H, base)[0]', '    q = rope(project(x_new, layer["Wq"])[None], [s - 1], H, base)[0]')),
    ("new key not rotated with s", ('layer["Wk"], layer["Wv"], H, base, pos0=s))', 'layer["Wk"], layer["Wv"], H, base, pos0=0))')),
    ("values rotated too", ("    v = project(X_head, Wv)\n", "    v = rope(project(X_head, Wv), np.arange(pos0, pos0 + l), n_heads, base)\n")),
    ("RMSNorm subtracts the mean", ("    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps) * _f64(g)", "    x = x - x.mean(axis=-1, keepdims=True)\n    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps) * _f64(g)")),
    ("sigmoid of the wrong sign", ("    return x / (1.0 + np.exp(-x))", "    return x / (1.0 + np.exp(x))")),
    ("gate and up exchanged", ("return project(silu(project(x, Wg)) * project(x, Wu), Wd)", "return project(silu(project(x, Wu)) * project(x, Wg), Wd)")),
]


def test_llama_unmutated_passes():
    assert llama_pins_hold(_load(LLAMA))


@pytest.mark.parametrize("name,replace", LLAMA_MUTATIONS, ids=[m[0] for m in LLAMA_MUTATIONS])
def test_llama_pins_catch(name, replace):
    assert not llama_pins_hold(_load(LLAMA, replace)), name


# ---- greedy sampling step ----
def greedy_pins_hold(ko) -> bool:
    try:
        hidden = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])
        W_lm = np.array([[1.0, 5.0, 5.0, 0.0], [2.0, 0.0, 7.0, 7.0]])
        emb = np.array([[10.0, 11.0], [20.0, 21.0], [30.0, 31.0], [40.0, 41.0]])
        tokens, logits, x_next = ko.greedy_next(hidden, W_lm, emb)
        return bool(np.array_equal(logits, [[1, 5, 5, 0], [2, 0, 7, 7], [3, 5, 12, 7]]) and tokens.tolist() == [1, 2, 2]
                    and np.array_equal(x_next, [[20, 21], [30, 31], [30, 31]]))
    except Exception:
        return False


ORACLE = os.path.join(ROOT, "oracle", "kvpr_oracle.py")
GREEDY_MUTATIONS = [
    ("last maximum on ties", ("    tokens = np.argmax(logits, axis=-1)", "    tokens = logits.shape[-1] - 1 - np.argmax(logits[..., ::-1], axis=-1)")),
    ("embedding row by batch index", ("_f64(emb)[tokens])", "_f64(emb)[: len(tokens)])")),
    ("argmin", ("    tokens = np.argmax(logits, axis=-1)", "    tokens = np.argmin(logits, axis=-1)")),
]


def test_greedy_unmutated_passes():
    assert greedy_pins_hold(_load(ORACLE))


@pytest.mark.parametrize("name,replace", GREEDY_MUTATIONS, ids=[m[0] for m in GREEDY_MUTATIONS])
def test_greedy_pins_catch(name, replace):
    assert not greedy_pins_hold(_load(ORACLE, replace)), name


# ---- wiring of the LLaMA-shaped decoder layer and stack, against the Hugging Face layer ----
def llama_stack_pins_hold(lo) -> bool:
    try:
        import test_oracle_llama_hf as hf
        cfg, layers = hf._hf_layers(2, 7)
        b, s = 2, 9
        hidden = torch.randn(b, s + 1, hf.H_DIM, dtype=torch.float64, generator=torch.Generator().manual_seed(8))
        h1, h2 = hf._run_hf(cfg, layers, hidden)
        with torch.no_grad():
            x1 = layers[0].input_layernorm(hidden).numpy()
            x2 = layers[1].input_layernorm(h1).numpy()
        Ls = [hf._as_oracle_layer(layers[0], np.ascontiguousarray(np.swapaxes(x1[:, :s], 0, 1))),
              hf._as_oracle_layer(layers[1], np.ascontiguousarray(np.swapaxes(x2[:, :s], 0, 1)))]
        one, _ = lo.decoder_stack_decode(Ls[:1], hidden[:, s].numpy(), [4], None, "none", "none")
        two, _ = lo.decoder_stack_decode(Ls, hidden[:, s].numpy(), [4, 9], None, "none", "none")
        return hf._close(one, h1[:, s].numpy()) and hf._close(two, h2[:, s].numpy())
    except Exception:
        return False


LLAMA_STACK_MUTATIONS = [
    ("attention residual dropped", ('        x = rnd(x + rnd(r["o"]))', '        x = rnd(rnd(r["o"]))')),
    ("FFN residual dropped", ('        x = rnd(x + rnd(project(f1, L["Wd"])))', '        x = rnd(rnd(project(f1, L["Wd"])))')),
    ("attention input not normalised", ('        xn = rnd(rms_norm(x, L["ln1_g"]))', "        xn = rnd(x)")),
    ("norm gains exchanged", ('        xn2 = rnd(rms_norm(x, L["ln2_g"]))', '        xn2 = rnd(rms_norm(x, L["ln1_g"]))')),
    ("second norm taken before the attention residual", ('        x = rnd(x + rnd(r["o"]))\n        xn2 = rnd(rms_norm(x, L["ln2_g"]))',
                                                         '        xn2 = rnd(rms_norm(x, L["ln2_g"]))\n        x = rnd(x + rnd(r["o"]))')),
    ("post-norm: the norm applied to the sum", ('        x = rnd(x + rnd(r["o"]))', '        x = rnd(rms_norm(x + rnd(r["o"]), L["ln2_g"]))')),
    ("every layer fed the stack input", ('        xn = rnd(rms_norm(x, L["ln1_g"]))', '        xn = rnd(rms_norm(_f64(x_in), L["ln1_g"]))')),
    ("silu on the up branch", ("        f1 = rnd(silu(g) * u)", "        f1 = rnd(g * silu(u))")),
]


def test_llama_stack_unmutated_passes():
    assert llama_stack_pins_hold(_load(LLAMA))


@pytest.mark.parametrize("name,replace", LLAMA_STACK_MUTATIONS, ids=[m[0] for m in LLAMA_STACK_MUTATIONS])
def test_llama_stack_pins_catch(name, replace):
    assert not llama_stack_pins_hold(_load(LLAMA, replace)), name
