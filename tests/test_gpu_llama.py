"""GPU parity of the LLaMA-shaped variant: rotary recompute GEMM, rotary token projection, the attention
layer at many splits (with and without chunked activation copies and the 4-bit store), the decoder stack
with RMSNorm and the gated FFN, and the column schedule."""
import numpy as np
import pytest
import torch

import kvpr_inputs
from oracle import kvpr_int4_oracle as qo
from oracle import kvpr_llama_oracle as lo
from oracle import kvpr_oracle as ko
from kvpr_testlib import dev, rel_err, rel_err_rms

pytestmark = pytest.mark.gpu
TOL = 1e-2
TIGHT = 3e-3


@pytest.fixture(scope="module")
def k():
    import paper_2411_17089_amd as k
    return k


@pytest.mark.parametrize("l,b,h,H,pos0", [(77, 3, 256, 4, 0), (9, 32, 512, 4, 5), (300, 1, 768, 12, 100), (40, 5, 256, 2, 1)])
def test_rotary_recompute_gemm_matches_oracle(k, l, b, h, H, pos0):
    print(f"rope gemm l={l} b={b} h={h} H={H} pos0={pos0}", flush=True)
    d = h // H
    lay = kvpr_inputs.make_layer(40 + l, b, l, h, H)
    n_pos = pos0 + l + 3
    table = dev(k.kvpr_rope_table(n_pos, d), torch.float32)
    wkv = dev(np.concatenate([lay["Wk"].T, lay["Wv"].T], 0))
    out = torch.full((l * b, 2 * h), float("nan"), dtype=torch.float16, device="cuda")
    k.kvpr_recompute_gemm_rope(dev(lay["X"]), wkv, None, out, l * b, 2 * h, h, 2 * h, table, n_pos, h, d, b, pos0)
    torch.cuda.synchronize()
    want = lo.recompute_kv(lay["X"], lay["Wk"], lay["Wv"], H, pos0=pos0).reshape(l * b, 2 * h)
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    assert rel_err(got[:, :h], want[:, :h]) <= 2e-3 and rel_err(got[:, h:], want[:, h:]) <= 2e-3
    # the value half is the plain GEMM's, bit for bit
    plain = torch.empty_like(out)
    k.kvpr_recompute_gemm(dev(lay["X"]), wkv, None, plain, l * b, 2 * h, h, 2 * h)
    torch.cuda.synchronize()
    assert torch.equal(plain[:, h:], out[:, h:])
    # rows beyond the table are refused on the host
    with pytest.raises(k.KvprError) as e:
        k.kvpr_recompute_gemm_rope(dev(lay["X"]), wkv, None, out, l * b, 2 * h, h, 2 * h, table, pos0 + l - 1, h, d, b, pos0)
    assert e.value.code == k.KVPR_E_RANGE


def test_rotary_gemm_with_column_band_mapping(k):
    """The rotary epilogue under the mapping that gives every XCD a band of tile columns (8 tile columns here)."""
    l, b, h, H, pos0 = 50, 7, 1024, 8, 3
    d = h // H
    lay = kvpr_inputs.make_layer(77, b, l, h, H)
    table = dev(k.kvpr_rope_table(pos0 + l, d), torch.float32)
    wkv = dev(np.concatenate([lay["Wk"].T, lay["Wv"].T], 0))
    want = lo.recompute_kv(lay["X"], lay["Wk"], lay["Wv"], H, pos0=pos0).reshape(l * b, 2 * h)
    for mapping in (1, 0):
        out = torch.full((l * b, 2 * h), float("nan"), dtype=torch.float16, device="cuda")
        k.lib.kvpr_debug_set_gemm_mapping(mapping)
        try:
            k.kvpr_recompute_gemm_rope(dev(lay["X"]), wkv, None, out, l * b, 2 * h, h, 2 * h, table, pos0 + l, h, d, b, pos0)
            torch.cuda.synchronize()
        finally:
            k.lib.kvpr_debug_set_gemm_mapping(-1)
        assert rel_err(out.cpu().numpy(), want) <= 2e-3, mapping


def test_rotary_token_projection_matches_oracle(k):
    b, h, H, pos = 5, 512, 4, 37
    rng = np.random.default_rng(3)
    qk = rng.standard_normal((b, 2 * h)).astype(np.float32)
    table = dev(k.kvpr_rope_table(pos + 1, h // H), torch.float32)
    q32 = torch.empty((b, h), dtype=torch.float32, device="cuda")
    row = torch.zeros((b, 2 * h), dtype=torch.float16, device="cuda")
    k.kvpr_rope_token(dev(qk, torch.float32), table, pos + 1, pos, b, h, h // H, q32, row, 2 * h)
    torch.cuda.synchronize()
    want_q = lo.rope(qk[None, :, :h], [pos], H)[0]
    want_k = lo.rope(qk[None, :, h:], [pos], H)[0]
    assert rel_err(q32.cpu().numpy(), want_q) <= 1e-6
    assert rel_err(row.cpu().numpy()[:, :h], want_k) <= 1e-3
    assert not row.cpu().numpy()[:, h:].any()


class LRig:
    def __init__(self, k, seed, b, s, h, H, max_seq=None, dtype_flags=0):
        self.k, self.b, self.s, self.h, self.H = k, b, s, h, H
        self.layer = kvpr_inputs.make_layer(seed, b, s, h, H)
        self.stored = lo.stored_kv(self.layer, "fp16").astype(np.float16)
        L = self.layer
        self.wqkv = dev(np.concatenate([L["Wq"].T, L["Wk"].T, L["Wv"].T], 0))
        self.wo = dev(L["Wo"].T)
        self.x_new = dev(L["x_new"])
        self.w = k.make_weights(wqkv=self.wqkv, wo=self.wo)
        self.ctx = k.kvpr_create(1, h, H, h // H, 0, b, max_seq or s + 2, dtype=k.KVPR_F16 | dtype_flags, arch=k.KVPR_ARCH_LLAMA)
        k.kvpr_store_write(self.ctx, 0, 0, s, np.ascontiguousarray(L["X"]), np.ascontiguousarray(self.stored))
        self.out = torch.empty((b, h), dtype=torch.float16, device="cuda")

    def decode(self, l, seq=None, x_new=None):
        self.k.kvpr_layer_decode(self.ctx, 0, self.s if seq is None else seq, l, self.w, self.x_new if x_new is None else x_new, self.out, False)
        torch.cuda.synchronize()
        return self.out.cpu().numpy().copy()

    def close(self):
        self.k.kvpr_destroy(self.ctx)


def test_small_config_every_eighth_split(k):
    rig = LRig(k, 0, 1, 128, 768, 12)
    try:
        ref = lo.layer_decode(rig.layer, 0, rig.stored)["o"]
        outs = []
        for l in list(range(0, 129, 8)) + [1, 127]:
            print(f"llama small split {l}", flush=True)
            o = rig.decode(l)
            outs.append(o)
            assert rel_err(o, ref) <= TIGHT and rel_err_rms(o, ref) <= TOL, l
        assert max(rel_err(o, outs[0]) for o in outs) <= 2e-3
        # the rotation matters: the OPT-shaped oracle without biases is far away
        plain = ko.layer_decode(dict(rig.layer, bq=None, bk=None, bv=None, bo=None), 0)["o"]
        assert rel_err(outs[0], plain) > 0.05
    finally:
        rig.close()


@pytest.mark.parametrize("seed,b,s,h,H", [(1, 3, 77, 256, 2), (2, 32, 40, 512, 4), (3, 5, 300, 768, 12), (5, 33, 20, 256, 4)])
def test_layer_decode_shapes_chunks_and_second_token(k, seed, b, s, h, H):
    rig = LRig(k, seed, b, s, h, H, max_seq=s + 3)
    try:
        ref = lo.layer_decode(rig.layer, 0, rig.stored)
        for chunks in (1, 3):
            k.kvpr_set_chunks(rig.ctx, chunks)
            for l in sorted({0, 1, s // 2, s - 1, s}):
                print(f"llama b={b} s={s} h={h} chunks={chunks} split {l}", flush=True)
                assert rel_err(rig.decode(l), ref["o"]) <= TIGHT, (chunks, l)
        k.kvpr_set_chunks(rig.ctx, 1)
        # second token: row s of the store was written by the first step (rotated with position s)
        x2 = kvpr_inputs._draw(np.random.default_rng(70 + seed), (b, h), 1.0)
        lay2 = dict(rig.layer, X=np.concatenate([rig.layer["X"], rig.layer["x_new"][None]], 0), x_new=x2)
        ref2 = lo.layer_decode(lay2, 0, np.concatenate([rig.stored.astype(np.float64), ref["kv"][s:s + 1]], 0))["o"]
        for l in (0, s // 3, s + 1):
            assert rel_err(rig.decode(l, seq=s + 1, x_new=dev(x2)), ref2) <= TIGHT, l
    finally:
        rig.close()


def test_rotary_layer_over_the_4bit_store(k):
    b, s, h, H = 4, 72, 256, 2
    rig = LRig(k, 8, b, s, h, H, dtype_flags=k.KVPR_STORE_INT4)
    try:
        kv_hat = qo.roundtrip(rig.stored).astype(np.float64)
        lay = dict(rig.layer, X=qo.roundtrip(rig.layer["X"]).astype(np.float64))
        for l in (0, 16, 40, s):
            assert rel_err(rig.decode(l), lo.layer_decode(lay, l, kv_hat)["o"]) <= TOL, l
    finally:
        rig.close()


def _llama_params(seed, b, h, H, ffn):
    P = kvpr_inputs.make_layer(seed, b, 1, h, H)
    P.update(kvpr_inputs.make_gated_ffn(seed, h, ffn))
    return P


def _lib_arrays(P):
    """Host arrays in the library's layouts: W stored [out, in], q|k|v fused, gate|up stacked."""
    arrs = {
        "wqkv": np.concatenate([P["Wq"].T, P["Wk"].T, P["Wv"].T], 0), "wo": P["Wo"].T,
        "w1": np.concatenate([P["Wg"].T, P["Wu"].T], 0), "w2": P["Wd"].T, "ln1_g": P["ln1_g"], "ln2_g": P["ln2_g"],
    }
    return {n: np.ascontiguousarray(a, dtype=np.float16) for n, a in arrs.items()}


def test_decoder_stack_and_columns(k):
    n_layers, nb, b, s, h, H, ffn = 3, 2, 4, 40, 256, 2, 768
    params = [_llama_params(600 + j, b, h, H, ffn) for j in range(n_layers)]
    layers = [[dict(params[j], X=kvpr_inputs._draw(np.random.default_rng([600, j, q]), (s, b, h), 1.0)) for q in range(nb)]
              for j in range(n_layers)]
    stored = [[lo.stored_kv(layers[j][q], "fp16").astype(np.float16) for q in range(nb)] for j in range(n_layers)]
    x_in = kvpr_inputs._draw(np.random.default_rng(599), (nb, b, h), 1.0)

    def oracle(q, splits):
        return lo.decoder_stack_decode([layers[j][q] for j in range(n_layers)], x_in[q], splits,
                                       [stored[j][q] for j in range(n_layers)])[0]

    ctx = k.kvpr_create(n_layers, h, H, h // H, ffn, b, s + 2, arch=k.KVPR_ARCH_LLAMA)
    try:
        keep, ws = [], []
        for j in range(n_layers):
            d = {n: dev(a) for n, a in _lib_arrays(params[j]).items()}
            keep.append(d)
            ws.append(k.make_weights(**d))
            k.kvpr_store_write(ctx, j, 0, s, np.ascontiguousarray(layers[j][0]["X"]), stored[j][0])
        out = torch.empty((b, h), dtype=torch.float16, device="cuda")
        for splits in ([0, 0, 0], [s, s, s], [7, 25, 40]):
            print(f"llama stack splits={splits}", flush=True)
            k.kvpr_decode_step(ctx, s, ws, dev(x_in[0]), out, splits)
            torch.cuda.synchronize()
            assert rel_err(out.cpu().numpy(), oracle(0, splits)) <= 5e-3
    finally:
        k.kvpr_destroy(ctx)

    ctx = k.kvpr_create_offload(n_layers, h, H, h // H, ffn, b, s + 2, nb, arch=k.KVPR_ARCH_LLAMA)
    try:
        keep = []
        for j in range(n_layers):
            arrs = _lib_arrays(params[j])
            keep.append(arrs)
            k.kvpr_weights_write(ctx, j, k.make_weights(**arrs))
            for q in range(nb):
                k.kvpr_store_write(ctx, j * nb + q, 0, s, np.ascontiguousarray(layers[j][q]["X"]), stored[j][q])
        x_out = torch.empty((nb, b, h), dtype=torch.float16, device="cuda")
        splits = [5, 40, 0, 16, 33, 24]
        print(f"llama columns splits={splits}", flush=True)
        k.kvpr_decode_step_columns(ctx, s, n_layers * nb, dev(x_in), x_out, splits)
        torch.cuda.synchronize()
        got = x_out.cpu().numpy()
        for q in range(nb):
            assert rel_err(got[q], oracle(q, [splits[j * nb + q] for j in range(n_layers)])) <= 5e-3, q
    finally:
        k.kvpr_destroy(ctx)


def test_prefill_helper_rotates(k):
    rig = LRig(k, 12, 4, 50, 256, 2)
    try:
        k.kvpr_store_prefill_kv(rig.ctx, 0, 50, rig.w)
        ref = lo.layer_decode(rig.layer, 0, rig.stored)["o"]
        assert rel_err(rig.decode(0), ref) <= TIGHT
    finally:
        rig.close()
