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
