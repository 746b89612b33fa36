"""Pin for the oracle's decoder-stack function: the last position of a causal forward pass of
torch's own pre-LayerNorm Transformer encoder layers (float64, CPU) over the s+1 tokens."""
import numpy as np
import pytest
import torch

from oracle import kvpr_oracle as ko


@pytest.mark.parametrize("n_layers,b,s,h,H,ffn", [(2, 2, 6, 16, 2, 32), (3, 1, 9, 24, 3, 40)])
def test_stack_is_last_row_of_causal_transformer(n_layers, b, s, h, H, ffn):
    torch.manual_seed(n_layers * 100 + s)
    tl = [torch.nn.TransformerEncoderLayer(h, H, ffn, dropout=0.0, activation="relu", norm_first=True,
                                           dtype=torch.float64) for _ in range(n_layers)]
    for layer in tl:                                     # non-trivial LayerNorm and bias parameters
        for p in layer.parameters():
            if p.dim() == 1:
                p.data = torch.randn_like(p) * 0.3 + (1.0 if p is layer.norm1.weight or p is layer.norm2.weight else 0.0)
    tokens = torch.randn(s + 1, b, h, dtype=torch.float64)
    mask = torch.nn.Transformer.generate_square_subsequent_mask(s + 1, dtype=torch.float64)
    ln1_out = []
    hooks = [layer.norm1.register_forward_hook(lambda m, i, o: ln1_out.append(o.detach().numpy().copy())) for layer in tl]
    x = tokens
    with torch.no_grad():
        for layer in tl:
            layer.train()                                 # keeps the plain (hookable) path; dropout is 0
            x = layer(x, src_mask=mask)
    for hk in hooks:
        hk.remove()
    want = x[-1].numpy()

    layers = []
    for i, layer in enumerate(tl):
        g = lambda t: t.detach().numpy()
        Wi, bi = g(layer.self_attn.in_proj_weight), g(layer.self_attn.in_proj_bias)
        layers.append({
            "n_heads": H, "X": ln1_out[i][:s],          # what the cached positions fed to W in this layer
            "Wq": Wi[:h].T, "Wk": Wi[h:2 * h].T, "Wv": Wi[2 * h:].T, "bq": bi[:h], "bk": bi[h:2 * h], "bv": bi[2 * h:],
            "Wo": g(layer.self_attn.out_proj.weight).T, "bo": g(layer.self_attn.out_proj.bias),
            "W1": g(layer.linear1.weight).T, "b1": g(layer.linear1.bias), "W2": g(layer.linear2.weight).T, "b2": g(layer.linear2.bias),
            "ln1_g": g(layer.norm1.weight), "ln1_b": g(layer.norm1.bias), "ln2_g": g(layer.norm2.weight), "ln2_b": g(layer.norm2.bias),
        })
    for splits in ([0] * n_layers, [s] * n_layers, [s // 2] * n_layers):
        got, trace = ko.decoder_stack_decode(layers, tokens[-1].numpy(), splits, kv_round="none", act_round="none")
        np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
        for i in range(n_layers):
            np.testing.assert_allclose(trace[i]["xn"], ln1_out[i][s], rtol=1e-10, atol=1e-12)


def test_activation_rounding_mode_is_close():
    rng = np.random.default_rng(3)
    h, H, ffn, s, b = 32, 2, 64, 5, 2
    L = {"n_heads": H, "X": rng.standard_normal((s, b, h))}
    for n, shape, sc in (("Wq", (h, h), .1), ("Wk", (h, h), .1), ("Wv", (h, h), .1), ("Wo", (h, h), .1), ("W1", (h, ffn), .1),
                         ("W2", (ffn, h), .1), ("bq", (h,), .1), ("bk", (h,), .1), ("bv", (h,), .1), ("bo", (h,), .1),
                         ("b1", (ffn,), .1), ("b2", (h,), .1), ("ln1_b", (h,), .1), ("ln2_b", (h,), .1)):
        L[n] = rng.standard_normal(shape) * sc
    L["ln1_g"] = np.ones(h)
    L["ln2_g"] = np.ones(h)
    x = rng.standard_normal((b, h))
    a, _ = ko.decoder_stack_decode([L, L], x, [2, 3], kv_round="none", act_round="none")
    c, _ = ko.decoder_stack_decode([L, L], x, [2, 3], kv_round="fp16", act_round="fp16")
    assert np.max(np.abs(a - c)) <= 5e-3 * np.max(np.abs(a))
    assert not np.array_equal(a, c)


def test_greedy_next_hand_values():
    """Greedy sampling step (row argmax of hidden . W_lm, lowest index on ties, embedding row of the token): a hand case
    with ties in two rows and a vocabulary wider than the hidden size, so that W_lm's orientation [h, vocab] is fixed."""
    hidden = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])
    W_lm = np.array([[1.0, 5.0, 5.0, 0.0],
                     [2.0, 0.0, 7.0, 7.0]])                         # [h = 2, vocab = 4]
    emb = np.array([[10.0, 11.0], [20.0, 21.0], [30.0, 31.0], [40.0, 41.0]])
    tokens, logits, x_next = ko.greedy_next(hidden, W_lm, emb)
    assert np.array_equal(logits, [[1, 5, 5, 0], [2, 0, 7, 7], [3, 5, 12, 7]])
    assert tokens.tolist() == [1, 2, 2]                             # rows 0 and 1 tie: the lower index wins
    assert np.array_equal(x_next, [[20, 21], [30, 31], [30, 31]])
    assert ko.greedy_next(hidden, W_lm)[2] is None
    with pytest.raises(ValueError):
        ko.greedy_next(hidden, W_lm.T)                              # [vocab, h] does not multiply a [b, h] hidden state
    # float16 inputs are taken at their exact values: a logit gap of one float16 ulp decides the token
    h16 = np.array([[1.0, 1.0]], dtype=np.float16)
    w16 = np.array([[1.0, 1.0], [1.0, np.float16(1.0) + np.float16(2.0 ** -10)]], dtype=np.float16)
    assert ko.greedy_next(h16, w16)[0].tolist() == [1]
