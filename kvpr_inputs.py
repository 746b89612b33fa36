"""Seeded synthetic inputs for one OPT-shaped decoder attention layer.

This module only draws random numbers and shapes them; it contains none of the
method's arithmetic (no projection, no attention, no cost model), so both the
CPU oracle's tests and the HIP path's tests/bench can share it without sharing
any computation.

Recipe (stand-in for the paper's workload of uniformly padded prompts fed to
OPT models, Experiments / "Workload"): every prompt in a batch has the same
length s, so a batch is a dense [s, b, h] block with no mask.
  X      [s, b, h]  ~ N(0, 1)      attention-input activations (token-major)
  x_new  [b, h]     ~ N(0, 1)      the decode token's attention input
  Wq, Wk, Wv, Wo  [h, h] ~ N(0, 0.02)   in the paper's orientation  y = x . W  (Eq. 1, Eq. 3)
  bq, bk, bv, bo  [h]    ~ N(0, 0.01)
All values are drawn in float32 from numpy's PCG64 stream seeded with `seed`,
scaled, then rounded to float16: the fp16 values ARE the inputs for both sides.
"""
from __future__ import annotations

import numpy as np

# name -> (hidden, heads, head_dim); OPT-shaped attention layers used by the configs.
SHAPES = {
    "tiny": (768, 12, 64),
    "opt-6.7b": (4096, 32, 128),
    "opt-13b": (5120, 40, 128),
    "opt-30b": (7168, 56, 128),
    "llama2-7b": (4096, 32, 128),
    "llama2-13b": (5120, 40, 128),
}
# gated-FFN width of the LLaMA-2 shapes
LLAMA_FFN = {"llama2-7b": 11008, "llama2-13b": 13824}


def _draw(rng: np.random.Generator, shape, scale: float) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    a *= np.float32(scale)
    return a.astype(np.float16)


def make_layer(seed: int, b: int, s: int, h: int, n_heads: int,
               w_scale: float = 0.02, b_scale: float = 0.01) -> dict:
    """Inputs of one attention layer. Draw order is fixed (weights first, so
    that the same seed gives the same weights for any b and s)."""
    if h % n_heads:
        raise ValueError("hidden must be a multiple of n_heads")
    rng = np.random.default_rng(seed)
    out = {"b": b, "s": s, "h": h, "n_heads": n_heads, "seed": seed}
    for name in ("Wq", "Wk", "Wv", "Wo"):
        out[name] = _draw(rng, (h, h), w_scale)
    for name in ("bq", "bk", "bv", "bo"):
        out[name] = _draw(rng, (h,), b_scale)
    out["x_new"] = _draw(rng, (b, h), 1.0)
    out["X"] = _draw(rng, (s, b, h), 1.0)
    return out


def make_ffn(seed: int, h: int, ffn: int, w_scale: float = 0.02, b_scale: float = 0.01) -> dict:
    """Extra parameters of a full OPT-style decoder layer: two LayerNorms and
    the two FFN matrices (Eq. 4), again in y = x . W orientation."""
    rng = np.random.default_rng([seed, 0xFF17])
    out = {"ffn": ffn}
    out["W1"] = _draw(rng, (h, ffn), w_scale)
    out["W2"] = _draw(rng, (ffn, h), w_scale)
    out["b1"] = _draw(rng, (ffn,), b_scale)
    out["b2"] = _draw(rng, (h,), b_scale)
    for name in ("ln1_g", "ln2_g"):
        out[name] = (np.float32(1.0) + rng.standard_normal((h,), dtype=np.float32) * np.float32(0.05)).astype(np.float16)
    for name in ("ln1_b", "ln2_b"):
        out[name] = _draw(rng, (h,), 0.02)
    return out


def make_gated_ffn(seed: int, h: int, ffn: int, w_scale: float = 0.02) -> dict:
    """Extra parameters of a LLaMA-style decoder layer: two RMSNorm gains and the gate / up / down
    matrices of the gated FFN, in y = x . W orientation."""
    rng = np.random.default_rng([seed, 0x11A3A])
    out = {"ffn": ffn}
    out["Wg"] = _draw(rng, (h, ffn), w_scale)
    out["Wu"] = _draw(rng, (h, ffn), w_scale)
    out["Wd"] = _draw(rng, (ffn, h), w_scale)
    for name in ("ln1_g", "ln2_g"):
        out[name] = (np.float32(1.0) + rng.standard_normal((h,), dtype=np.float32) * np.float32(0.05)).astype(np.float16)
    return out
