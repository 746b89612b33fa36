"""Pins of the LLaMA-shaped oracle against the implementation the paper ran LLaMA-2 on (appendix "Additional Experimental
Results on LLaMa Models": the Hugging Face transformers LlamaDecoderLayer): rotary embedding, RMSNorm, the wiring of one
decoder layer, and the composition of two layers.  The layers are built in code from a small LlamaConfig with random
weights, in float64, eager attention, on the CPU; nothing is downloaded."""
import numpy as np
import pytest
import torch

from oracle import kvpr_llama_oracle as lo

tf = pytest.importorskip("transformers")
from transformers import LlamaConfig  # noqa: E402
from transformers.models.llama.modeling_llama import (LlamaDecoderLayer, LlamaRMSNorm, LlamaRotaryEmbedding,  # noqa: E402
                                                      apply_rotary_pos_emb)

H_DIM, HEADS, FFN, EPS = 128, 2, 256, 1e-5


def _close(got, want, tol=5e-6):
    """max |got - want| / max |want|: the Hugging Face modules normalise and form cos / sin in float32 (about 2e-7 here);
    a dropped residual, a swapped norm or a wrong rotation is a difference of order 0.1."""
    return float(np.max(np.abs(np.asarray(got) - np.asarray(want))) / np.max(np.abs(np.asarray(want)))) <= tol


def _config():
    cfg = LlamaConfig(hidden_size=H_DIM, intermediate_size=FFN, num_hidden_layers=2, num_attention_heads=HEADS,
                      num_key_value_heads=HEADS, rms_norm_eps=EPS, rope_theta=10000.0, attention_bias=False, mlp_bias=False,
                      max_position_embeddings=512, vocab_size=32, attention_dropout=0.0)
    cfg._attn_implementation = "eager"
    return cfg


def _hf_layers(n, seed):
    torch.manual_seed(seed)
    cfg = _config()
    layers = [LlamaDecoderLayer(cfg, i).double().eval() for i in range(n)]
    for lay in layers:                                         # norm gains away from 1 so that a dropped gain shows
        with torch.no_grad():
            lay.input_layernorm.weight.copy_(1.0 + 0.3 * torch.randn(H_DIM, dtype=torch.float64))
            lay.post_attention_layernorm.weight.copy_(1.0 + 0.3 * torch.randn(H_DIM, dtype=torch.float64))
            for p in (lay.self_attn.q_proj, lay.self_attn.k_proj, lay.self_attn.v_proj, lay.self_attn.o_proj,
                      lay.mlp.gate_proj, lay.mlp.up_proj, lay.mlp.down_proj):
                p.weight.copy_(0.2 * torch.randn_like(p.weight))
    return cfg, layers


def _as_oracle_layer(lay, X_post_norm):
    """Weights in the oracle's orientation (y = x . W) and the cached post-norm activations [s, b, h]."""
    w = lambda lin: lin.weight.detach().numpy().T.copy()
    return {"Wq": w(lay.self_attn.q_proj), "Wk": w(lay.self_attn.k_proj), "Wv": w(lay.self_attn.v_proj),
            "Wo": w(lay.self_attn.o_proj), "Wg": w(lay.mlp.gate_proj), "Wu": w(lay.mlp.up_proj), "Wd": w(lay.mlp.down_proj),
            "ln1_g": lay.input_layernorm.weight.detach().numpy().copy(),
            "ln2_g": lay.post_attention_layernorm.weight.detach().numpy().copy(),
            "n_heads": HEADS, "X": X_post_norm, "x_new": None}


def _run_hf(cfg, layers, hidden):
    """Causal forward of hidden [b, S, h] through the layers; returns the list of per-layer outputs."""
    b, S, _ = hidden.shape
    pos = torch.arange(S)[None].expand(b, S)
    cos, sin = LlamaRotaryEmbedding(cfg)(hidden, pos)
    mask = torch.full((S, S), float("-inf"), dtype=torch.float64).triu(1)[None, None].expand(b, 1, S, S)
    outs = []
    x = hidden
    with torch.no_grad():
        for lay in layers:
            x = lay(x, attention_mask=mask, position_ids=pos, position_embeddings=(cos.double(), sin.double()))
            x = x[0] if isinstance(x, tuple) else x
            outs.append(x)
    return outs


def test_rope_and_rmsnorm_match_the_hugging_face_modules():
    cfg = _config()
    rng = np.random.default_rng(0)
    b, S, d = 3, 9, H_DIM // HEADS
    q = rng.standard_normal((b, S, H_DIM))
    kx = rng.standard_normal((b, S, H_DIM))
    pos = torch.tensor([[0, 1, 2, 3, 10, 57, 58, 300, 511]]).expand(b, S)
    cos, sin = LlamaRotaryEmbedding(cfg)(torch.from_numpy(q), pos)
    heads = lambda a: torch.from_numpy(a).reshape(b, S, HEADS, d).transpose(1, 2)
    qe, ke = apply_rotary_pos_emb(heads(q), heads(kx), cos.double(), sin.double())
    back = lambda t: t.transpose(1, 2).reshape(b, S, H_DIM).numpy()
    # the oracle takes [P, ..., h] with one position per leading row: positions are shared by the batch
    mine_q = lo.rope(np.swapaxes(q, 0, 1), pos[0].numpy(), HEADS)
    mine_k = lo.rope(np.swapaxes(kx, 0, 1), pos[0].numpy(), HEADS)
    # HF forms the angle p * theta in float32: its error grows like p * 6e-8 (3e-5 rad at p = 511); a wrong pairing,
    # sign, exponent or position is an O(1) difference
    assert np.allclose(np.swapaxes(mine_q, 0, 1), back(qe), rtol=0, atol=2e-4)
    assert np.allclose(np.swapaxes(mine_k, 0, 1), back(ke), rtol=0, atol=2e-4)
    small = slice(0, 4)                                                   # positions 0..3: float32 angles are exact enough
    assert np.allclose(np.swapaxes(mine_q, 0, 1)[:, small], back(qe)[:, small], rtol=0, atol=1e-6)
    norm = LlamaRMSNorm(H_DIM, eps=EPS).double()
    with torch.no_grad():
        norm.weight.copy_(torch.from_numpy(rng.standard_normal(H_DIM)))
        want = norm(torch.from_numpy(q)).numpy()
    assert np.allclose(lo.rms_norm(q, norm.weight.detach().numpy(), EPS), want, rtol=1e-6, atol=1e-7)   # HF normalises in float32


@pytest.mark.parametrize("split", [0, 5, 11])
def test_one_decoder_layer_is_the_last_row_of_the_hugging_face_layer(split):
    """Decode of token s with the first `split` cache rows recomputed = row s of a causal forward over s + 1 tokens."""
    cfg, (lay,) = _hf_layers(1, 3)
    b, s = 2, 11
    hidden = torch.randn(b, s + 1, H_DIM, dtype=torch.float64, generator=torch.Generator().manual_seed(4))
    want = _run_hf(cfg, [lay], hidden)[0][:, s].numpy()
    with torch.no_grad():
        xn_all = lay.input_layernorm(hidden).numpy()                       # what the method stores: the post-norm activations
    L = _as_oracle_layer(lay, np.ascontiguousarray(np.swapaxes(xn_all[:, :s], 0, 1)))
    got, _ = lo.decoder_stack_decode([L], hidden[:, s].numpy(), [split], None, "none", "none")
    assert _close(got, want)


def test_two_decoder_layers_compose_like_the_hugging_face_stack():
    cfg, layers = _hf_layers(2, 7)
    b, s = 2, 9
    hidden = torch.randn(b, s + 1, H_DIM, dtype=torch.float64, generator=torch.Generator().manual_seed(8))
    h1, h2 = _run_hf(cfg, layers, hidden)
    with torch.no_grad():
        x1 = layers[0].input_layernorm(hidden).numpy()
        x2 = layers[1].input_layernorm(h1).numpy()                         # layer 2's cached activations come from its prefill
    Ls = [_as_oracle_layer(layers[0], np.ascontiguousarray(np.swapaxes(x1[:, :s], 0, 1))),
          _as_oracle_layer(layers[1], np.ascontiguousarray(np.swapaxes(x2[:, :s], 0, 1)))]
    got, trace = lo.decoder_stack_decode(Ls, hidden[:, s].numpy(), [4, 9], None, "none", "none")
    assert _close(got, h2[:, s].numpy())
    # the second layer saw the first layer's output for the new token, normalised with its own gain
    assert _close(trace[1]["xn"], x2[:, s])
