"""CPU oracle for KVPR's per-layer decode path.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this file.  It shares no code with the HIP library and never imports it.

KVPR reaches exactly the result of plain decode attention (Introduction: exact
attention, no approximation), so the oracle is the plain definition written out
in numpy float64, one function per equation of the paper:

  Eq. 1  (Background)          Q = X.Wq, K = X.Wk, V = X.Wv
  Eq. 2  (Background)          Z = softmax(Q.K^T / sqrt(d_head)).V   per head
  Eq. 3  (Background)          O = Z.Wo
  Eq. 4  (Background)          FFN  sigma(O.W1).W2
  Eq. 5  (Background)          decode: K,V <- concat(K,V ; x.Wk, x.Wv)
  Eq. 7  (Scheduler Module)    recompute K[0:l] = X[0:l].Wk, V[0:l] = X[0:l].Wv
  Sec. 3.2, "partial recomputation": the GPU merges recomputed rows [0,l) with
                               transferred rows [l,s)

Readings where the paper is silent:
  * projections carry a bias (OPT has one); bias 0 gives the paper's equations;
  * heads are contiguous blocks of d_head columns; softmax subtracts the row max;
  * no mask: the one new token attends to all s+1 positions;
  * layout is token-major: X[s, b, h], KV[s, b, 2h] with a row = [K(h) | V(h)];
  * kv_round="fp16" rounds every K/V row (stored, recomputed, new) to float16
    before attention, modelling a float16 KV cache; everything else is float64.
    kv_round="none" rounds nothing.

Every function is pinned by tests/test_oracle_*.py (closed forms, a hand-worked
example, textbook special cases via torch CPU, brute force).  Nothing here is
"parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=F64)


def round_fp16(a: np.ndarray) -> np.ndarray:
    """Round to nearest-even float16 and return as float64."""
    return _f64(a).astype(np.float16).astype(F64)


# --------------------------------------------------------------------------
# Eq. 1 / Eq. 3 / Eq. 7: a projection is rows . W (+ bias)
# --------------------------------------------------------------------------
def project(x: np.ndarray, W: np.ndarray, bias=None) -> np.ndarray:
    """y[..., n] = sum_k x[..., k] * W[k, n] + bias[n]   (paper orientation x.W)."""
    y = _f64(x) @ _f64(W)
    if bias is not None:
        y = y + _f64(bias)
    return y


def recompute_kv(X_head: np.ndarray, Wk, Wv, bk=None, bv=None) -> np.ndarray:
    """Eq. 7: K and V of the first l positions from their activations.

    X_head [l, b, h]  ->  [l, b, 2h] whose rows are [K | V].
    """
    K = project(X_head, Wk, bk)
    V = project(X_head, Wv, bv)
    return np.concatenate([K, V], axis=-1)


def full_kv(X, Wk, Wv, bk=None, bv=None) -> np.ndarray:
    """Eq. 1 restricted to K and V, all s positions: what prefill stores."""
    return recompute_kv(X, Wk, Wv, bk, bv)


def new_token_kv(x_new, Wk, Wv, bk=None, bv=None) -> np.ndarray:
    """Eq. 5: the decode token's own K/V row, [b, 2h]."""
    return np.concatenate([project(x_new, Wk, bk), project(x_new, Wv, bv)], axis=-1)


def assemble_kv(l: int, X, kv_stored, x_new, Wk, Wv, bk=None, bv=None,
                kv_round: str = "fp16") -> np.ndarray:
    """The KV the attention sees for split l: [s+1, b, 2h].

    rows [0, l)  recomputed from X[0:l]         (Eq. 7)
    rows [l, s)  taken from the stored cache    (the transferred part)
    row  s       the new token's K/V            (Eq. 5)
    """
    X = _f64(X)
    s = X.shape[0]
    if not 0 <= l <= s:
        raise ValueError(f"split {l} outside [0, {s}]")
    parts = [recompute_kv(X[:l], Wk, Wv, bk, bv),
             _f64(kv_stored)[l:s],
             new_token_kv(x_new, Wk, Wv, bk, bv)[None]]
    kv = np.concatenate(parts, axis=0)
    if kv_round == "fp16":
        kv = round_fp16(kv)
    elif kv_round != "none":
        raise ValueError(kv_round)
    return kv


# --------------------------------------------------------------------------
# Eq. 2: decode attention of one query per sequence over s+1 positions
# --------------------------------------------------------------------------
def decode_attention(q: np.ndarray, kv: np.ndarray, n_heads: int) -> np.ndarray:
    """q [b, h], kv [S, b, 2h] -> z [b, h].

    For sequence n and head i (columns [i*d, (i+1)*d)):
      score_j = q[n, head i] . K[j, n, head i] / sqrt(d),  p = softmax_j(score),
      z[n, head i] = sum_j p_j V[j, n, head i].
    """
    q = _f64(q)
    kv = _f64(kv)
    b, h = q.shape
    S = kv.shape[0]
    d = h // n_heads
    K = kv[:, :, :h].reshape(S, b, n_heads, d)
    V = kv[:, :, h:].reshape(S, b, n_heads, d)
    qh = q.reshape(b, n_heads, d)
    scores = np.einsum("bid,jbid->bij", qh, K) / math.sqrt(d)
    scores = scores - scores.max(axis=-1, keepdims=True)
    p = np.exp(scores)
    p = p / p.sum(axis=-1, keepdims=True)
    z = np.einsum("bij,jbid->bid", p, V)
    return z.reshape(b, h)


def layer_decode(layer: dict, l: int, kv_stored=None, kv_round: str = "fp16") -> dict:
    """One decode step of one attention layer at split l.

    `layer` holds X, x_new, Wq..Wo, bq..bo, n_heads (see kvpr_inputs.make_layer).
    `kv_stored` is the host cache [s, b, 2h]; if None it is what prefill would
    have stored, full_kv(X) rounded like the cache.
    Returns q, kv (assembled, s+1 rows), z and o = z.Wo + bo (Eq. 3).
    """
    if kv_stored is None:
        kv_stored = stored_kv(layer, kv_round)
    kv = assemble_kv(l, layer["X"], kv_stored, layer["x_new"], layer["Wk"], layer["Wv"],
                     layer["bk"], layer["bv"], kv_round)
    q = project(layer["x_new"], layer["Wq"], layer["bq"])
    z = decode_attention(q, kv, layer["n_heads"])
    o = project(z, layer["Wo"], layer["bo"])
    return {"q": q, "kv": kv, "z": z, "o": o}


def stored_kv(layer: dict, kv_round: str = "fp16") -> np.ndarray:
    """The cache prefill leaves on the host: Eq. 1's K,V for every prompt position."""
    kv = full_kv(layer["X"], layer["Wk"], layer["Wv"], layer["bk"], layer["bv"])
    return round_fp16(kv) if kv_round == "fp16" else kv


# --------------------------------------------------------------------------
# The same layer, written a second time as scalar loops with exactly rounded
# sums (math.fsum of float64 products; products of two float16 values are exact
# in float64).  Only for tiny shapes: it cross-checks the indexing of the numpy
# version and makes "recompute == stored" and "output independent of l" hold
# bit for bit.
# --------------------------------------------------------------------------
def _dot(u, v) -> float:
    return math.fsum(float(a) * float(c) for a, c in zip(u, v))


def layer_decode_loops(layer: dict, l: int, kv_stored=None) -> dict:
    X, x_new = _f64(layer["X"]), _f64(layer["x_new"])
    Wq, Wk, Wv, Wo = (_f64(layer[n]) for n in ("Wq", "Wk", "Wv", "Wo"))
    bq, bk, bv, bo = (_f64(layer[n]) for n in ("bq", "bk", "bv", "bo"))
    s, b, h = X.shape
    H = layer["n_heads"]
    d = h // H

    def kv_row(x):  # Eq. 7 / Eq. 5 for one token of one sequence
        k = [_dot(x, Wk[:, n]) + bk[n] for n in range(h)]
        v = [_dot(x, Wv[:, n]) + bv[n] for n in range(h)]
        return k + v

    o = np.zeros((b, h))
    z = np.zeros((b, h))
    kv = np.zeros((s + 1, b, 2 * h))
    for n in range(b):
        for j in range(s + 1):
            if j < l:
                kv[j, n] = kv_row(X[j, n])
            elif j < s:
                kv[j, n] = kv_stored[j, n] if kv_stored is not None else kv_row(X[j, n])
            else:
                kv[j, n] = kv_row(x_new[n])
        q = [_dot(x_new[n], Wq[:, c]) + bq[c] for c in range(h)]
        for i in range(H):
            cols = range(i * d, (i + 1) * d)
            sc = [_dot([q[c] for c in cols], [kv[j, n, c] for c in cols]) / math.sqrt(d)
                  for j in range(s + 1)]
            m = max(sc)
            e = [math.exp(v - m) for v in sc]
            tot = math.fsum(e)
            for c in cols:
                z[n, c] = math.fsum(e[j] * kv[j, n, h + c] for j in range(s + 1)) / tot
        for c in range(h):
            o[n, c] = _dot(z[n], Wo[:, c]) + bo[c]
    return {"kv": kv, "z": z, "o": o}


# --------------------------------------------------------------------------
# Rest of an OPT-style decoder layer (Eq. 4 plus the LayerNorms and residuals
# the paper leaves to the model): used only by the layer-stack checks.
# --------------------------------------------------------------------------
def layer_norm(x, g, beta, eps: float = 1e-5) -> np.ndarray:
    x = _f64(x)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * _f64(g) + _f64(beta)


def ffn(o, W1, b1, W2, b2) -> np.ndarray:
    """Eq. 4 with sigma = ReLU (OPT) and biases."""
    return project(np.maximum(project(o, W1, b1), 0.0), W2, b2)


def decoder_stack_decode(layers, x_in, splits, stored=None, kv_round: str = "fp16", act_round: str = "fp16"):
    """One decode token through a stack of OPT-style decoder layers (Sec. 4 "Implementation":
    row-by-row schedule, one batch, layer after layer).

    Each entry of `layers` holds the attention parameters and X of kvpr_inputs.make_layer plus the
    FFN / LayerNorm parameters of kvpr_inputs.make_ffn.  Per layer:
        xn = LN1(x);  o = attention block at split l on (X, stored KV, x_new = xn);  x = x + o;
        x = x + FFN(LN2(x))                                                      (Eq. 4, ReLU)
    act_round="fp16" rounds every activation tensor the runtime keeps in float16 (xn, o, the
    residual sums, the FFN hidden and output) at the point where it is stored; all arithmetic
    in between is float64.  Returns the final hidden state and the per-layer (xn, new K|V row).
    """
    rnd = round_fp16 if act_round == "fp16" else _f64
    x = _f64(x_in)
    trace = []
    for i, L in enumerate(layers):
        xn = rnd(layer_norm(x, L["ln1_g"], L["ln1_b"]))
        att = dict(L)
        att["x_new"] = xn
        kv_st = stored[i] if stored is not None else None
        r = layer_decode(att, splits[i], kv_st, kv_round)
        o = rnd(r["o"])
        x = rnd(x + o)
        xn2 = rnd(layer_norm(x, L["ln2_g"], L["ln2_b"]))
        f1 = rnd(np.maximum(project(xn2, L["W1"], L["b1"]), 0.0))
        f2 = rnd(project(f1, L["W2"], L["b2"]))
        x = rnd(x + f2)
        trace.append({"xn": xn, "kv_new": r["kv"][-1]})
    return x, trace


def greedy_next(hidden, W_lm, emb=None):
    """Greedy sampling: logits = hidden . W_lm (W_lm [h, vocab]), token = first argmax,
    next input = embedding row.  Returns (tokens, logits, x_next or None)."""
    logits = project(hidden, W_lm)
    tokens = np.argmax(logits, axis=-1)
    return tokens, logits, (None if emb is None else _f64(emb)[tokens])
