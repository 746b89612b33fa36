"""CPU oracle for the group-wise 4-bit KV-cache codec.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this file.
It shares no code with the HIP library and never imports it.

The paper (Sec. 4.4, "KV Cache Compression") says only that the transferred cache is compressed
with group-wise 4-bit quantization; it fixes neither the group shape nor the rounding.  The
reading implemented here:

  * a group is 64 consecutive columns of one row of one sequence: a cache row [K(h) | V(h)], or, when
    the stored activations are compressed as well, an activation row X(h).  Compressing only the
    cache would make a position's activations (2h bytes) dearer to send than its compressed cache
    (9h/8 bytes) and Eq. 10 would then never choose to recompute, so the same codec is applied to
    both by default (9h/16 bytes per activation row);
  * asymmetric min/max quantisation: mn = min(group), mx = max(group),
        scale = float16((mx - mn) / 15)         (float32 arithmetic, then rounded to float16)
        code  = clip(rint((x - mn) / scale), 0, 15)   (float32, round-half-to-even; 0 if scale == 0)
        xhat  = float16(code * scale + mn)      (float32 multiply, float32 add, then float16)
    mn is itself a float16 value of the group, so it is stored exactly;
  * a compressed row of c columns is  [c/2 bytes of codes | c/64 pairs (scale, mn) of float16]:
    element 2k of a row sits in the low nibble of byte k, element 2k+1 in the high nibble.
    9c/16 bytes per row instead of 2c.

The integer codes are decided in float32 on both sides (here with numpy float32 operations, one
IEEE operation each), so they can be compared bit for bit with the GPU's.
"""
from __future__ import annotations

import numpy as np

GROUP = 64


def packed_bytes(cols: int) -> int:
    """Bytes of one compressed row of `cols` columns (cols a multiple of 64)."""
    if cols % GROUP:
        raise ValueError("cols must be a multiple of 64")
    return cols // 2 + (cols // GROUP) * 4


def quantize_rows(kv: np.ndarray):
    """kv [..., c] float16  ->  codes uint8 [..., c] (values 0..15), scale float16 [..., c/64], mn float16 [..., c/64]."""
    kv = np.asarray(kv, dtype=np.float16)
    g = kv.reshape(kv.shape[:-1] + (kv.shape[-1] // GROUP, GROUP)).astype(np.float32)
    mn = g.min(axis=-1)
    mx = g.max(axis=-1)
    scale16 = ((mx - mn) / np.float32(15.0)).astype(np.float16)
    scale = scale16.astype(np.float32)
    safe = np.where(scale > 0, scale, np.float32(1.0))
    q = np.rint((g - mn[..., None]) / safe[..., None])
    q = np.where(scale[..., None] > 0, q, np.float32(0.0))
    codes = np.clip(q, 0, 15).astype(np.uint8)
    return codes.reshape(kv.shape), scale16, mn.astype(np.float16)


def dequantize_rows(codes: np.ndarray, scale16: np.ndarray, mn16: np.ndarray) -> np.ndarray:
    """Inverse map, float16 result."""
    c = codes.reshape(codes.shape[:-1] + (codes.shape[-1] // GROUP, GROUP)).astype(np.float32)
    prod = c * scale16.astype(np.float32)[..., None]                      # float32 multiply
    x = (prod + mn16.astype(np.float32)[..., None]).astype(np.float16)    # float32 add, then float16
    return x.reshape(codes.shape)


def pack_rows(codes: np.ndarray, scale16: np.ndarray, mn16: np.ndarray) -> np.ndarray:
    """The byte layout of compressed rows: uint8 [..., packed_bytes(c)]."""
    lo = codes[..., 0::2]
    hi = codes[..., 1::2]
    nib = (lo | (hi << 4)).astype(np.uint8)
    meta = np.stack([scale16, mn16], axis=-1).astype(np.float16)          # [..., groups, 2]
    meta_bytes = meta.reshape(meta.shape[:-2] + (-1,)).view(np.uint8)
    return np.concatenate([nib, meta_bytes], axis=-1)


def unpack_rows(packed: np.ndarray, cols: int):
    h = cols // 2
    nib = packed[..., :h]
    codes = np.empty(packed.shape[:-1] + (2 * h,), dtype=np.uint8)
    codes[..., 0::2] = nib & 15
    codes[..., 1::2] = nib >> 4
    meta = np.ascontiguousarray(packed[..., h:]).view(np.float16).reshape(packed.shape[:-1] + (2 * h // GROUP, 2))
    return codes, meta[..., 0], meta[..., 1]


def roundtrip(kv: np.ndarray) -> np.ndarray:
    """What the attention sees for a transferred row: dequantize(quantize(row)), float16."""
    return dequantize_rows(*quantize_rows(kv))


def layer_decode_int4(layer: dict, l: int, compress_x: bool = True, kv_stored=None):
    """One attention layer's decode step over a compressed host store (Sec. 4.4 on top of Sec. 3.2).

    Rows [l, s) of the cache are what the store returns, dequantize(quantize(KV)); rows [0, l) are
    recomputed (Eq. 7) from what the store returns for the activations, dequantize(quantize(X)) when
    they are compressed too; the new token's row (Eq. 5) is exact.  kv_stored (float16 values,
    [s, b, 2h]) overrides the prefill cache that is compressed.
    """
    from oracle import kvpr_oracle as ko

    kv = ko.stored_kv(layer, "fp16") if kv_stored is None else np.asarray(kv_stored)
    kv_hat = roundtrip(kv.astype(np.float16)).astype(np.float64)
    lay = dict(layer)
    if compress_x:
        lay["X"] = roundtrip(np.asarray(layer["X"]).astype(np.float16)).astype(np.float64)
    return ko.layer_decode(lay, l, kv_hat, "fp16")
