"""CPU oracle for the LLaMA-shaped variant of the decode path.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this file.
It shares no code with the HIP library and never imports it.

The paper evaluates LLaMA-2 7B / 13B with the same method (Experiments, first paragraph; appendix
"Additional Experimental Results on LLaMa Models") and says only that the attention mechanism is
similar.  What differs from the OPT-shaped layer, and the readings taken here:

  * no biases in the projections;
  * rotary position embedding on q and k.  The cache holds K *after* rotation, so the partial
    recomputation (Eq. 7) must rotate the recomputed rows with their own positions:
        K[0:l] = RoPE(X[0:l] . Wk, positions 0 .. l-1),   V[0:l] = X[0:l] . Wv
    and the decode token's q and k (Eq. 1, Eq. 5) are rotated with position s.
    Convention: the half-split pairing of the Hugging Face implementation the paper builds on:
    within a head of width d, element i pairs with element i + d/2,
        theta_i = base^(-2i/d),  i = 0 .. d/2 - 1,  base = 10000
        y[i]       = x[i] cos(p theta_i) - x[i + d/2] sin(p theta_i)
        y[i + d/2] = x[i + d/2] cos(p theta_i) + x[i] sin(p theta_i)
    All sequences of a batch share positions (uniformly padded prompts, as in the paper's workload);
  * RMSNorm (eps 1e-5, no offset) in place of LayerNorm;
  * gated FFN: down( silu(x . Wg) * (x . Wu) ) in place of Eq. 4's two-matrix ReLU FFN.

Rounding model (as in the OPT oracle): float64 arithmetic; kv_round="fp16" rounds every K/V row
to float16 where the cache stores it (after the rotation).
"""
from __future__ import annotations

import numpy as np

from oracle.kvpr_oracle import _f64, decode_attention, project, round_fp16


def rope_angles(positions, d: int, base: float = 10000.0) -> np.ndarray:
    """p * theta_i for every position p and i in [0, d/2): shape [len(positions), d/2]."""
    i = np.arange(d // 2, dtype=np.float64)
    theta = base ** (-2.0 * i / d)
    return np.asarray(positions, dtype=np.float64)[:, None] * theta[None, :]


def rope(x: np.ndarray, positions, n_heads: int, base: float = 10000.0) -> np.ndarray:
    """Rotate x [P, ..., h] (P = len(positions), heads contiguous in the last axis) by its positions."""
    x = _f64(x)
    h = x.shape[-1]
    d = h // n_heads
    ang = rope_angles(positions, d, base)                                   # [P, d/2]
    shape = (x.shape[0],) + (1,) * (x.ndim - 2) + (1, d // 2)
    c, s = np.cos(ang).reshape(shape), np.sin(ang).reshape(shape)
    xh = x.reshape(x.shape[:-1] + (n_heads, d))
    x1, x2 = xh[..., : d // 2], xh[..., d // 2:]
    out = np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)
    return out.reshape(x.shape)


def recompute_kv(X_head: np.ndarray, Wk, Wv, n_heads: int, base: float = 10000.0, pos0: int = 0) -> np.ndarray:
    """Eq. 7 for a rotary model: rows [pos0, pos0 + l) of the cache from their activations."""
    l = X_head.shape[0]
    k = rope(project(X_head, Wk), np.arange(pos0, pos0 + l), n_heads, base)
    v = project(X_head, Wv)
    return np.concatenate([k, v], axis=-1)


def stored_kv(layer: dict, kv_round: str = "fp16") -> np.ndarray:
    kv = recompute_kv(layer["X"], layer["Wk"], layer["Wv"], layer["n_heads"], layer.get("rope_base", 10000.0))
    return round_fp16(kv) if kv_round == "fp16" else kv


def layer_decode(layer: dict, l: int, kv_stored=None, kv_round: str = "fp16") -> dict:
    """One decode step of one rotary attention layer at split l (no biases)."""
    X, x_new, H = layer["X"], layer["x_new"], layer["n_heads"]
    base = layer.get("rope_base", 10000.0)
    s = X.shape[0]
    if not 0 <= l <= s:
        raise ValueError("split outside [0, s]")
    if kv_stored is None:
        kv_stored = stored_kv(layer, kv_round)
    rnd = round_fp16 if kv_round == "fp16" else _f64
    head = rnd(recompute_kv(X[:l], layer["Wk"], layer["Wv"], H, base))      # recomputed rows
    tail = _f64(kv_stored)[l:s]                                             # transferred rows
    new = rnd(recompute_kv(_f64(x_new)[None], layer["Wk"], layer["Wv"], H, base, pos0=s))   # Eq. 5 at position s
    kv = np.concatenate([head, tail, new], axis=0)
    q = rope(project(x_new, layer["Wq"])[None], [s], H, base)[0]
    z = decode_attention(q, kv, H)
    o = project(z, layer["Wo"])
    return {"q": q, "kv": kv, "z": z, "o": o}


def rms_norm(x, g, eps: float = 1e-5) -> np.ndarray:
    x = _f64(x)
    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps) * _f64(g)


def silu(x) -> np.ndarray:
    x = _f64(x)
    return x / (1.0 + np.exp(-x))


def gated_ffn(x, Wg, Wu, Wd) -> np.ndarray:
    return project(silu(project(x, Wg)) * project(x, Wu), Wd)


def decoder_stack_decode(layers, x_in, splits, stored=None, kv_round: str = "fp16", act_round: str = "fp16"):
    """One decode token through a stack of LLaMA-style decoder layers:
        xn = RMSNorm1(x); x = x + attention block(xn); x = x + down(silu(gate(RMSNorm2(x))) * up(RMSNorm2(x)))
    act_round="fp16" rounds every activation tensor the runtime keeps in float16 where it is stored
    (the two normalised inputs, o, the residual sums, the gate|up projections, their gated product,
    the FFN output)."""
    rnd = round_fp16 if act_round == "fp16" else _f64
    x = _f64(x_in)
    trace = []
    for i, L in enumerate(layers):
        xn = rnd(rms_norm(x, L["ln1_g"]))
        att = dict(L)
        att["x_new"] = xn
        r = layer_decode(att, splits[i], stored[i] if stored is not None else None, kv_round)
        x = rnd(x + rnd(r["o"]))
        xn2 = rnd(rms_norm(x, L["ln2_g"]))
        g, u = rnd(project(xn2, L["Wg"])), rnd(project(xn2, L["Wu"]))
        f1 = rnd(silu(g) * u)
        x = rnd(x + rnd(project(f1, L["Wd"])))
        trace.append({"xn": xn, "kv_new": r["kv"][-1]})
    return x, trace
