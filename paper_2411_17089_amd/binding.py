"""ctypes binding of libkvpr.so: same names as include/kvpr.h, argument marshalling only.

Device arguments are torch CUDA tensors (or raw integer addresses); the binding passes
their data_ptr().  Nothing is computed here and there is no fallback: if the library is
missing the import fails.
"""
from __future__ import annotations

import ctypes as C
import os

# torch ships its own HIP runtime; load it first so that libkvpr.so binds to the same runtime
# instance that owns torch's device memory and streams (two runtimes in one process do not mix).
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvpr.so")

KVPR_OK, KVPR_E_INVAL, KVPR_E_RANGE, KVPR_E_NOMEM, KVPR_E_HIP, KVPR_E_STATE = 0, -1, -2, -3, -4, -5
KVPR_F16 = 1
KVPR_KV_INT4, KVPR_X_INT4, KVPR_STORE_INT4 = 0x100, 0x200, 0x300
KVPR_COST_EQ10, KVPR_COST_NS, KVPR_COST_ROW, KVPR_COST_PIPE = 0, 1, 2, 3
KVPR_DEBUG_SYNC, KVPR_DEBUG_POISON = 1, 2
KVPR_ARCH_OPT, KVPR_ARCH_LLAMA = 0, 1
KVPR_ATTENTION_STATIC_SCRATCH_BYTES = 2 << 20


class kvpr_model_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "hidden", "n_heads", "head_dim", "ffn_dim", "batch", "max_seq", "dtype", "arch")] + [("rope_base", C.c_float)]


class kvpr_profile_t(C.Structure):
    _fields_ = [(n, C.c_double) for n in
                ("h2d_bytes_per_s", "gemm_flops_per_s", "h2d_latency_s", "gemm_latency_s",
                 "d2h_bytes_per_s", "attn_bytes_per_s", "h2d_peak_bytes_per_s", "gemm_alone_flops_per_s")] + \
               [("gemm_round_flops", C.c_int64), ("layer_other_s", C.c_double)]


class kvpr_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("wqkv", "bqkv", "wo", "bo", "ln1_g", "ln1_b", "w1", "b1", "w2", "b2", "ln2_g", "ln2_b")]


class kvpr_layer_timing(C.Structure):
    _fields_ = [(n, C.c_float) for n in
                ("ms_act_copy", "ms_kv_copy", "ms_recompute", "ms_proj", "ms_attn", "ms_out", "ms_store",
                 "ms_assemble", "ms_total")] + [("t_bound_s", C.c_double), ("split", C.c_int32), ("ms_attn_early", C.c_float),
                                     ("ms_recompute_start", C.c_float), ("ms_weights_landed", C.c_float),
                                     ("weights_landed_valid", C.c_int32)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class KvprError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"kvpr error {code}: {text}")
        self.code = code


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} not found: build it with `python paper_2411_17089_amd/build.py` "
                      "(there is no CPU fallback)")
lib = C.CDLL(LIB_PATH)

_vp, _i, _i64, _sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
_SIGS = {
    "kvpr_last_error": (C.c_char_p, []),
    "kvpr_create": (_i, [C.POINTER(kvpr_model_desc), _vp, C.POINTER(_vp)]),
    "kvpr_destroy": (_i, [_vp]),
    "kvpr_set_debug": (_i, [_vp, _i]),
    "kvpr_set_profile": (_i, [_vp, C.POINTER(kvpr_profile_t), _i, _i]),
    "kvpr_store_write": (_i, [_vp, _i, _i, _i, _vp, _vp]),
    "kvpr_store_ptrs": (_i, [_vp, _i, C.POINTER(_vp), C.POINTER(_vp)]),
    "kvpr_store_prefill_kv": (_i, [_vp, _i, _i, C.POINTER(kvpr_layer_weights)]),
    "kvpr_profile": (_i, [_vp, _i, _i, C.POINTER(kvpr_profile_t)]),
    "kvpr_profile_step": (_i, [_vp, _i, _i, C.POINTER(kvpr_profile_t)]),
    "kvpr_plan_split": (_i, [C.POINTER(kvpr_profile_t), _i, _i, _i, _i, _i, _i, C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
    "kvpr_cost": (_i, [C.POINTER(kvpr_profile_t), _i, _i, _i, _i, _i, _i, C.POINTER(C.c_double)]),
    "kvpr_set_chunks": (_i, [_vp, _i]),
    "kvpr_set_hidden_offload": (_i, [_vp, _i]),
    "kvpr_set_weight_pipeline": (_i, [_vp, _i]),
    "kvpr_cost_chunked": (_i, [C.POINTER(kvpr_profile_t), _i, _i, _i, _i, _i, _i, C.POINTER(C.c_double)]),
    "kvpr_plan_split_chunked": (_i, [C.POINTER(kvpr_profile_t), _i, _i, _i, _i, _i, _i, C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
    "kvpr_cost_linear": (_i, [C.POINTER(kvpr_profile_t), _i, _i, _i, _i, _i64, _i64, _i64, C.POINTER(C.c_double)]),
    "kvpr_plan_split_linear": (_i, [C.POINTER(kvpr_profile_t), _i, _i, _i, _i64, _i64, _i64, _i, C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
    "kvpr_adapt_update": (_i, [C.POINTER(kvpr_profile_t), C.c_double, _i64, C.c_double, _i64, C.c_double]),
    "kvpr_set_adaptive": (_i, [_vp, C.c_double]),
    "kvpr_get_profile": (_i, [_vp, C.POINTER(kvpr_profile_t)]),
    "kvpr_set_keep_warm": (_i, [_vp, C.c_double]),
    "kvpr_layer_decode": (_i, [_vp, _i, _i, _i, C.POINTER(kvpr_layer_weights), _vp, _vp, C.POINTER(kvpr_layer_timing)]),
    "kvpr_layer_decode_timed": (_i, [_vp, _i, _i, _i, C.POINTER(kvpr_layer_weights), _vp, _vp, _i]),
    "kvpr_timing_read": (_i, [_vp, _i, C.POINTER(kvpr_layer_timing)]),
    "kvpr_decode_step": (_i, [_vp, _i, C.POINTER(kvpr_layer_weights), _vp, _vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(kvpr_layer_timing)]),
    "kvpr_create_offload": (_i, [C.POINTER(kvpr_model_desc), _i, _vp, C.POINTER(_vp)]),
    "kvpr_weights_write": (_i, [_vp, _i, C.POINTER(kvpr_layer_weights)]),
    "kvpr_decode_step_columns": (_i, [_vp, _i, _vp, _vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(kvpr_layer_timing)]),
    "kvpr_greedy_next": (_i, [_vp, _vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp]),
    "kvpr_recompute_gemm": (_i, [_vp, _vp, _vp, _vp, _i64, _i, _i, _i64, _vp]),
    "kvpr_decode_attention": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp]),
    "kvpr_attention_workspace_bytes": (_sz, [_i, _i, _i, _i]),
    "kvpr_decode_attention_static": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _vp]),
    "kvpr_decode_attention_mixed": (_i, [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp]),
    "kvpr_token_gemm": (_i, [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i64, _vp]),
    "kvpr_token_gemm_workspace_bytes": (_sz, [_i, _i]),
    "kvpr_token_gemm_ws": (_i, [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i64, _vp, _sz, _vp]),
    "kvpr_rope_table": (_i, [_vp, _i, _i, C.c_double]),
    "kvpr_recompute_gemm_rope": (_i, [_vp, _vp, _vp, _vp, _i64, _i, _i, _i64, _vp, _i, _i, _i, _i, _i, _vp]),
    "kvpr_rope_token": (_i, [_vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _i64, _vp]),
    "kvpr_int4_row_bytes": (_sz, [_i]),
    "kvpr_quant_int4": (_i, [_vp, _vp, _i64, _i, _vp]),
    "kvpr_dequant_int4": (_i, [_vp, _vp, _i64, _i, _vp]),
}
EXPORTS = tuple(_SIGS)
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.restype, _f.argtypes = _res, _args


def _check(rc: int):
    if rc != KVPR_OK:
        raise KvprError(rc, lib.kvpr_last_error().decode())


def _ptr(t):
    """Address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    if hasattr(t, "ctypes"):
        return t.ctypes.data
    raise TypeError(type(t))


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def kvpr_last_error() -> str:
    return lib.kvpr_last_error().decode()


def kvpr_create(n_layers, hidden, n_heads, head_dim, ffn_dim, batch, max_seq, stream=None, dtype=KVPR_F16,
                arch=KVPR_ARCH_OPT, rope_base=0.0):
    d = kvpr_model_desc(n_layers, hidden, n_heads, head_dim, ffn_dim, batch, max_seq, dtype, arch, rope_base)
    out = _vp()
    _check(lib.kvpr_create(C.byref(d), _stream(stream), C.byref(out)))
    return out


def kvpr_destroy(ctx):
    _check(lib.kvpr_destroy(ctx))


def kvpr_set_debug(ctx, flags):
    _check(lib.kvpr_set_debug(ctx, flags))


def kvpr_set_profile(ctx, prof, cost_model=KVPR_COST_EQ10, granularity=1):
    _check(lib.kvpr_set_profile(ctx, C.byref(prof), cost_model, granularity))


def kvpr_store_write(ctx, layer, t0, t1, x_host=None, kv_host=None):
    _check(lib.kvpr_store_write(ctx, layer, t0, t1, _ptr(x_host), _ptr(kv_host)))


def kvpr_store_ptrs(ctx, layer):
    x, kv = _vp(), _vp()
    _check(lib.kvpr_store_ptrs(ctx, layer, C.byref(x), C.byref(kv)))
    return x.value, kv.value


def kvpr_store_prefill_kv(ctx, layer, seq, weights):
    _check(lib.kvpr_store_prefill_kv(ctx, layer, seq, C.byref(weights)))


def kvpr_profile(ctx, batch, seq) -> kvpr_profile_t:
    p = kvpr_profile_t()
    _check(lib.kvpr_profile(ctx, batch, seq, C.byref(p)))
    return p


def kvpr_profile_step(ctx, batch, seq, prof) -> kvpr_profile_t:
    """Returns a copy of prof with gemm_flops_per_s as one single-layer decode step runs the GEMM."""
    p = kvpr_profile_t.from_buffer_copy(prof)
    _check(lib.kvpr_profile_step(ctx, batch, seq, C.byref(p)))
    return p


def make_profile(v_com, v_gpu, lat_com=0.0, lat_gpu=0.0, other=0.0, round_flops=0) -> kvpr_profile_t:
    return kvpr_profile_t(v_com, v_gpu, lat_com, lat_gpu, 0.0, 0.0, 0.0, 0.0, round_flops, other)


def kvpr_plan_split(prof, cost_model, batch, seq, hidden, elem_bytes=2, granularity=1):
    l, t = C.c_int32(), C.c_double()
    _check(lib.kvpr_plan_split(C.byref(prof), cost_model, batch, seq, hidden, elem_bytes, granularity, C.byref(l), C.byref(t)))
    return l.value, t.value


def kvpr_cost(prof, cost_model, split, batch, seq, hidden, elem_bytes=2):
    t = C.c_double()
    _check(lib.kvpr_cost(C.byref(prof), cost_model, split, batch, seq, hidden, elem_bytes, C.byref(t)))
    return t.value


def kvpr_set_weight_pipeline(ctx, fine_grained):
    _check(lib.kvpr_set_weight_pipeline(ctx, int(fine_grained)))


def kvpr_set_hidden_offload(ctx, on):
    _check(lib.kvpr_set_hidden_offload(ctx, int(on)))


def kvpr_set_chunks(ctx, chunks):
    _check(lib.kvpr_set_chunks(ctx, chunks))


def kvpr_cost_chunked(prof, chunks, split, batch, seq, hidden, elem_bytes=2):
    t = C.c_double()
    _check(lib.kvpr_cost_chunked(C.byref(prof), chunks, split, batch, seq, hidden, elem_bytes, C.byref(t)))
    return t.value


def kvpr_plan_split_chunked(prof, chunks, batch, seq, hidden, elem_bytes=2, granularity=1):
    l, t = C.c_int32(), C.c_double()
    _check(lib.kvpr_plan_split_chunked(C.byref(prof), chunks, batch, seq, hidden, elem_bytes, granularity, C.byref(l), C.byref(t)))
    return l.value, t.value


def kvpr_cost_linear(prof, cost_model, chunks, split, seq, x_bytes_per_pos, kv_bytes_per_pos, flops_per_pos):
    t = C.c_double()
    _check(lib.kvpr_cost_linear(C.byref(prof), cost_model, chunks, split, seq, x_bytes_per_pos, kv_bytes_per_pos,
                                flops_per_pos, C.byref(t)))
    return t.value


def kvpr_plan_split_linear(prof, cost_model, chunks, seq, x_bytes_per_pos, kv_bytes_per_pos, flops_per_pos, granularity=1):
    l, t = C.c_int32(), C.c_double()
    _check(lib.kvpr_plan_split_linear(C.byref(prof), cost_model, chunks, seq, x_bytes_per_pos, kv_bytes_per_pos,
                                      flops_per_pos, granularity, C.byref(l), C.byref(t)))
    return l.value, t.value


def make_weights(**tensors) -> kvpr_layer_weights:
    """kvpr_layer_weights from device tensors given by field name; keeps no reference (caller keeps them alive)."""
    w = kvpr_layer_weights()
    for k, v in tensors.items():
        setattr(w, k, _ptr(v))
    return w


def kvpr_layer_decode(ctx, layer, seq, split, weights, x_new_dev, out_dev, timing=False):
    t = kvpr_layer_timing() if timing else None
    _check(lib.kvpr_layer_decode(ctx, layer, seq, split, C.byref(weights), _ptr(x_new_dev), _ptr(out_dev),
                                 C.byref(t) if timing else None))
    return t


def kvpr_layer_decode_timed(ctx, layer, seq, split, weights, x_new_dev, out_dev, slot):
    _check(lib.kvpr_layer_decode_timed(ctx, layer, seq, split, C.byref(weights), _ptr(x_new_dev), _ptr(out_dev), slot))


def kvpr_timing_read(ctx, slot) -> kvpr_layer_timing:
    t = kvpr_layer_timing()
    _check(lib.kvpr_timing_read(ctx, slot, C.byref(t)))
    return t


def kvpr_decode_step(ctx, seq, layer_weights, x_in_dev, x_out_dev, splits=None, timing=False):
    n = len(layer_weights)
    arr = (kvpr_layer_weights * n)(*layer_weights)
    sin = (C.c_int32 * n)(*splits) if splits is not None else None
    sout = (C.c_int32 * n)()
    tim = (kvpr_layer_timing * n)() if timing else None
    _check(lib.kvpr_decode_step(ctx, seq, arr, _ptr(x_in_dev), _ptr(x_out_dev), sin, sout, tim))
    return list(sout), (list(tim) if timing else None)


def kvpr_create_offload(n_layers, hidden, n_heads, head_dim, ffn_dim, batch, max_seq, n_gpu_batches, stream=None, dtype=KVPR_F16,
                        arch=KVPR_ARCH_OPT, rope_base=0.0):
    d = kvpr_model_desc(n_layers, hidden, n_heads, head_dim, ffn_dim, batch, max_seq, dtype, arch, rope_base)
    out = _vp()
    _check(lib.kvpr_create_offload(C.byref(d), n_gpu_batches, _stream(stream), C.byref(out)))
    return out


def kvpr_weights_write(ctx, layer, host_weights):
    _check(lib.kvpr_weights_write(ctx, layer, C.byref(host_weights)))


def kvpr_decode_step_columns(ctx, seq, n_slots, x_in_dev, x_out_dev, splits=None, timing=False):
    sin = (C.c_int32 * n_slots)(*splits) if splits is not None else None
    sout = (C.c_int32 * n_slots)()
    tim = (kvpr_layer_timing * n_slots)() if timing else None
    _check(lib.kvpr_decode_step_columns(ctx, seq, _ptr(x_in_dev), _ptr(x_out_dev), sin, sout, tim))
    return list(sout), (list(tim) if timing else None)


def kvpr_greedy_next(hidden_dev, w_lm_dev, emb_dev, batch, hidden, vocab, logits_dev, tokens_dev, x_next_dev, stream=None):
    _check(lib.kvpr_greedy_next(_ptr(hidden_dev), _ptr(w_lm_dev), _ptr(emb_dev), batch, hidden, vocab, _ptr(logits_dev),
                                _ptr(tokens_dev), _ptr(x_next_dev), _stream(stream)))


def kvpr_recompute_gemm(a_dev, w_dev, bias_dev, c_dev, M, N, K, ldc, stream=None):
    _check(lib.kvpr_recompute_gemm(_ptr(a_dev), _ptr(w_dev), _ptr(bias_dev), _ptr(c_dev), M, N, K, ldc, _stream(stream)))


def kvpr_attention_workspace_bytes(batch, hidden, n_heads, S) -> int:
    return lib.kvpr_attention_workspace_bytes(batch, hidden, n_heads, S)


def kvpr_decode_attention(q_dev, kv_dev, z_dev, ws_dev, S, batch, hidden, n_heads, stream=None):
    _check(lib.kvpr_decode_attention(_ptr(q_dev), _ptr(kv_dev), _ptr(z_dev), _ptr(ws_dev), S, batch, hidden, n_heads, _stream(stream)))


def kvpr_decode_attention_static(q_dev, kv_dev, z_dev, S, batch, hidden, n_heads, stream=None):
    _check(lib.kvpr_decode_attention_static(_ptr(q_dev), _ptr(kv_dev), _ptr(z_dev), S, batch, hidden, n_heads, _stream(stream)))


def kvpr_token_gemm(x_dev, w_dev, bias_dev, y32_dev, y16_dev, M, N, K, out_f32_cols, ld16, stream=None):
    _check(lib.kvpr_token_gemm(_ptr(x_dev), _ptr(w_dev), _ptr(bias_dev), _ptr(y32_dev), _ptr(y16_dev), M, N, K,
                               out_f32_cols, ld16, _stream(stream)))


def kvpr_token_gemm_workspace_bytes(M, N) -> int:
    return lib.kvpr_token_gemm_workspace_bytes(M, N)


def kvpr_token_gemm_ws(x_dev, w_dev, bias_dev, y32_dev, y16_dev, M, N, K, out_f32_cols, ld16, ws_dev, ws_bytes, stream=None):
    _check(lib.kvpr_token_gemm_ws(_ptr(x_dev), _ptr(w_dev), _ptr(bias_dev), _ptr(y32_dev), _ptr(y16_dev), M, N, K,
                                  out_f32_cols, ld16, _ptr(ws_dev), ws_bytes, _stream(stream)))


def kvpr_int4_row_bytes(cols) -> int:
    return lib.kvpr_int4_row_bytes(cols)


def kvpr_quant_int4(src_dev, dst_dev, rows, cols, stream=None):
    _check(lib.kvpr_quant_int4(_ptr(src_dev), _ptr(dst_dev), rows, cols, _stream(stream)))


def kvpr_dequant_int4(src_dev, dst_dev, rows, cols, stream=None):
    _check(lib.kvpr_dequant_int4(_ptr(src_dev), _ptr(dst_dev), rows, cols, _stream(stream)))


def kvpr_rope_table(n_pos, head_dim, base=10000.0):
    """numpy float32 [n_pos, head_dim/2, 2] = (cos, sin)."""
    import numpy as np
    out = np.empty((n_pos, head_dim // 2, 2), dtype=np.float32)
    _check(lib.kvpr_rope_table(out.ctypes.data, n_pos, head_dim, base))
    return out


def kvpr_recompute_gemm_rope(a_dev, w_dev, bias_dev, c_dev, M, N, K, ldc, table_dev, n_pos, rope_cols, head_dim, batch, pos0,
                             stream=None):
    _check(lib.kvpr_recompute_gemm_rope(_ptr(a_dev), _ptr(w_dev), _ptr(bias_dev), _ptr(c_dev), M, N, K, ldc, _ptr(table_dev),
                                        n_pos, rope_cols, head_dim, batch, pos0, _stream(stream)))


def kvpr_rope_token(qk32_dev, table_dev, n_pos, pos, batch, hidden, head_dim, q32_dev, k16_dev, ldk, stream=None):
    _check(lib.kvpr_rope_token(_ptr(qk32_dev), _ptr(table_dev), n_pos, pos, batch, hidden, head_dim, _ptr(q32_dev),
                               _ptr(k16_dev), ldk, _stream(stream)))


def kvpr_adapt_update(prof, alpha, link_bytes, link_seconds, gemm_flops, gemm_seconds):
    _check(lib.kvpr_adapt_update(C.byref(prof), alpha, link_bytes, link_seconds, gemm_flops, gemm_seconds))
    return prof


def kvpr_set_adaptive(ctx, alpha):
    _check(lib.kvpr_set_adaptive(ctx, alpha))


def kvpr_set_keep_warm(ctx, fraction):
    _check(lib.kvpr_set_keep_warm(ctx, fraction))


def kvpr_get_profile(ctx) -> kvpr_profile_t:
    p = kvpr_profile_t()
    _check(lib.kvpr_get_profile(ctx, C.byref(p)))
    return p


def kvpr_decode_attention_mixed(q_dev, kv16_dev, kvq_dev, z_dev, ws_dev, S, split, batch, hidden, n_heads, stream=None):
    _check(lib.kvpr_decode_attention_mixed(_ptr(q_dev), _ptr(kv16_dev), _ptr(kvq_dev), _ptr(z_dev), _ptr(ws_dev), S, split,
                                           batch, hidden, n_heads, _stream(stream)))
