"""Helpers shared by the GPU parity tests: move a synthetic layer to the device in the
library's layouts, and the error metrics.  No method arithmetic lives here."""
import numpy as np
import torch


def rel_err(got, ref) -> float:
    """max |got - ref| / max |ref|: the parity metric (1e-2 is the stated bar for fp16 with fp32 accumulate)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


def rel_err_rms(got, ref) -> float:
    """max element-wise error with the denominator floored at rms(ref)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    floor = np.sqrt(np.mean(ref ** 2)) + 1e-30
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)))


def dev(a, dtype=torch.float16):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda", dtype=dtype)


def upload_layer(layer: dict) -> dict:
    """Device tensors in the library's weight layout: W stored [out, in], q|k|v fused."""
    wqkv = np.concatenate([layer["Wq"].T, layer["Wk"].T, layer["Wv"].T], axis=0)
    bqkv = np.concatenate([layer["bq"], layer["bk"], layer["bv"]])
    out = {
        "wqkv": dev(wqkv), "bqkv": dev(bqkv),
        "wo": dev(layer["Wo"].T), "bo": dev(layer["bo"]),
        "x_new": dev(layer["x_new"]),
    }
    for k in ("ln1_g", "ln1_b", "ln2_g", "ln2_b", "b1", "b2"):
        if k in layer:
            out[k] = dev(layer[k])
    if "W1" in layer:
        out["w1"] = dev(layer["W1"].T)
        out["w2"] = dev(layer["W2"].T)
    return out
