"""Pins of the oracle's Transformer arithmetic against things other than itself:
closed forms, hand-computed cases, and the stock library Transformer as a special case.
CPU only."""
import math

import numpy as np
import pytest
import torch

from ad_inputs import init_weights, model_dims
from oracle import ad_oracle as O


def make(name="micro", seed=11, dtype=np.float64, contract=False, tie=False, std=0.02):
    dims = model_dims(name)
    w = init_weights(dims, seed, std=std, tie_output=tie)
    return dims, w, O.Model(dims, w, dtype, contract=contract, max_pos=64)


# ---------------------------------------------------------------- elementary pieces
def test_positions_closed_forms():
    d = 8
    pe = O.sinusoid_positions(5, d)
    # position 0: sin(0)=0 on even channels, cos(0)=1 on odd channels
    assert np.array_equal(pe[0], np.array([0, 1] * (d // 2), dtype=np.float64))
    # channel pair 0 has wavelength 2*pi: sin(p), cos(p)
    for p in range(5):
        assert pe[p, 0] == pytest.approx(math.sin(p), abs=1e-15)
        assert pe[p, 1] == pytest.approx(math.cos(p), abs=1e-15)
    # last pair: frequency 10000^-((d-2)/d)
    assert pe[3, d - 2] == pytest.approx(math.sin(3 * 10000 ** (-(d - 2) / d)), abs=1e-15)
    assert pe[3, d - 1] == pytest.approx(math.cos(3 * 10000 ** (-(d - 2) / d)), abs=1e-15)
    # the geometric progression of wavelengths from 2*pi to 10000*2*pi: pair i of d=4 is 10000^-(i/2)
    pe4 = O.sinusoid_positions(2, 4)
    assert pe4[1, 2] == pytest.approx(math.sin(0.01), abs=1e-15)


def test_layer_norm_hand_case():
    dims = dict(model_dims("nano"), d_model=4, n_heads=1)
    w = init_weights(dims, 1)
    w["enc.0.ln1.g"] = np.array([1, 2, 1, 1], dtype=np.float32)
    w["enc.0.ln1.b"] = np.array([0, 0, 0.5, 0], dtype=np.float32)
    m = O.Model(dims, w, np.float64, max_pos=4)
    y = m.layer_norm(np.array([[1.0, 2.0, 3.0, 4.0]]), "enc.0.ln1")
    s = math.sqrt(1.25 + 1e-5)  # biased variance of 1..4 is 1.25
    assert np.allclose(y[0], [-1.5 / s, 2 * -0.5 / s, 0.5 / s + 0.5, 1.5 / s], atol=1e-14)


def test_layer_norm_moments():
    dims, w, m = make()
    rng = np.random.default_rng(0)
    x = rng.normal(3.0, 5.0, size=(7, dims["d_model"]))
    m.p["enc.0.ln1.g"][:] = 1.0
    m.p["enc.0.ln1.b"][:] = 0.0
    y = m.layer_norm(x, "enc.0.ln1")
    assert np.allclose(y.mean(axis=1), 0, atol=1e-13)
    assert np.allclose(y.var(axis=1), 1, atol=1e-5)  # eps only


def test_attention_uniform_and_causal_closed_form():
    """Zero queries give equal weights: the output is the mean of the visible values."""
    dims, w, m = make()
    rng = np.random.default_rng(1)
    T, d = 6, dims["d_model"]
    k = rng.normal(size=(T, d))
    v = rng.normal(size=(T, d))
    out = m.attention(np.zeros((T, d)), k, v, [i + 1 for i in range(T)])
    for i in range(T):
        assert np.allclose(out[i], v[:i + 1].mean(axis=0), atol=1e-13)
    out = m.attention(np.zeros((T, d)), k, v, [T] * T)
    assert np.allclose(out, np.tile(v.mean(axis=0), (T, 1)), atol=1e-13)


def test_attention_selects_matching_key_per_head():
    """A query aligned with one key at a huge scale picks that key's value, head by head."""
    dims, w, m = make()
    d, H, dh = dims["d_model"], dims["n_heads"], dims["d_model"] // dims["n_heads"]
    T = 5
    k = np.zeros((T, d))
    v = np.arange(T * d, dtype=np.float64).reshape(T, d)
    q = np.zeros((1, d))
    pick = [3, 1]
    for h in range(H):
        for t in range(T):
            k[t, h * dh + t] = 1.0           # key t of head h = unit vector e_t
        q[0, h * dh + pick[h]] = 1e4         # query of head h points at key pick[h]
    out = m.attention(q, k, v, [T])
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        assert np.allclose(out[0, sl], v[pick[h], sl], atol=1e-9)


def test_attention_scale_is_inverse_sqrt_head_dim():
    """Two keys, one head slice: weights must be softmax(q.k / sqrt(dh))."""
    dims, w, m = make()
    d, dh = dims["d_model"], dims["d_model"] // dims["n_heads"]
    q = np.zeros((1, d)); k = np.zeros((2, d)); v = np.zeros((2, d))
    q[0, 0] = 2.0; k[0, 0] = 3.0; k[1, 0] = -1.0
    v[0, 0] = 1.0
    out = m.attention(q, k, v, [2])
    e0, e1 = math.exp(6.0 / math.sqrt(dh)), math.exp(-2.0 / math.sqrt(dh))
    assert out[0, 0] == pytest.approx(e0 / (e0 + e1), abs=1e-14)


def test_embed_scale_and_position():
    dims, w, m = make()
    x = m.embed([7, 9], [0, 3])
    d = dims["d_model"]
    expect0 = w["emb"][7].astype(np.float64) * math.sqrt(d) + np.array([0, 1] * (d // 2))
    assert np.allclose(x[0], expect0, atol=1e-14)
    assert x[1, 0] == pytest.approx(float(w["emb"][9, 0]) * math.sqrt(d) + math.sin(3.0), abs=1e-14)


def test_output_projection_tied_and_untied():
    dims, w, m = make(tie=False)
    x = np.random.default_rng(2).normal(size=(3, dims["d_model"]))
    assert np.allclose(m.logits(x), x @ w["out.w"].astype(np.float64).T, atol=1e-13)
    dims, w, m = make(tie=True)
    assert "out.w" not in w
    assert np.allclose(m.logits(x), x @ w["emb"].astype(np.float64).T, atol=1e-13)


def test_argmax_lowest_index_on_ties():
    assert O.argmax_lowest(np.array([1.0, 5.0, 5.0, 2.0])) == 1
    assert O.argmax_lowest(np.array([5.0, 5.0, 5.0])) == 0


# ---------------------------------------------------------------- bf16 rounding
def test_bf16_round_ties_to_even_hand_cases():
    one = np.float32(1.0)
    ulp = np.float32(2.0 ** -7)                      # bf16 spacing in [1,2)
    cases = {
        1.0: 1.0,
        1.0 + 2.0 ** -8: 1.0,                        # tie -> even mantissa (0)
        1.0 + 3 * 2.0 ** -8: 1.0 + 2 * 2.0 ** -7,    # tie -> even mantissa (2)
        1.0 + 2.0 ** -8 + 2.0 ** -20: 1.0 + 2.0 ** -7,  # just above the tie
        -3.0: -3.0,
        0.0: 0.0,
    }
    for x, y in cases.items():
        assert O.bf16_round(np.array([x], dtype=np.float32))[0] == np.float32(y), x
    assert ulp > 0 and one == 1


def test_bf16_round_matches_library_cast():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(O.bf16_round(x), ref)
    # float64 input goes through float32 first and keeps its dtype
    y = O.bf16_round(x.astype(np.float64))
    assert y.dtype == np.float64 and np.array_equal(y.astype(np.float32), ref)


# ---------------------------------------------------------------- whole stacks vs the stock library module
def _load_attn(mha, w, prefix):
    with torch.no_grad():
        mha.in_proj_weight.copy_(torch.from_numpy(np.concatenate([w[prefix + ".wq"], w[prefix + ".wk"], w[prefix + ".wv"]])))
        mha.in_proj_bias.copy_(torch.from_numpy(np.concatenate([w[prefix + ".bq"], w[prefix + ".bk"], w[prefix + ".bv"]])))
        mha.out_proj.weight.copy_(torch.from_numpy(w[prefix + ".wo"]))
        mha.out_proj.bias.copy_(torch.from_numpy(w[prefix + ".bo"]))


def _load_ffn_ln(layer, w, ffn, lns):
    with torch.no_grad():
        layer.linear1.weight.copy_(torch.from_numpy(w[ffn + ".w1"])); layer.linear1.bias.copy_(torch.from_numpy(w[ffn + ".b1"]))
        layer.linear2.weight.copy_(torch.from_numpy(w[ffn + ".w2"])); layer.linear2.bias.copy_(torch.from_numpy(w[ffn + ".b2"]))
        for norm, name in lns:
            norm.weight.copy_(torch.from_numpy(w[name + ".g"])); norm.bias.copy_(torch.from_numpy(w[name + ".b"]))


def _torch_stacks(dims, w):
    d, H, F = dims["d_model"], dims["n_heads"], dims["d_ffn"]
    kw = dict(d_model=d, nhead=H, dim_feedforward=F, dropout=0.0, activation="relu",
              layer_norm_eps=1e-5, batch_first=True, norm_first=False, dtype=torch.float64)
    enc = torch.nn.TransformerEncoder(torch.nn.TransformerEncoderLayer(**kw), dims["enc_layers"],
                                      enable_nested_tensor=False)
    dec = torch.nn.TransformerDecoder(torch.nn.TransformerDecoderLayer(**kw), dims["dec_layers"])
    for l, layer in enumerate(enc.layers):
        _load_attn(layer.self_attn, w, f"enc.{l}.self")
        _load_ffn_ln(layer, w, f"enc.{l}.ffn", [(layer.norm1, f"enc.{l}.ln1"), (layer.norm2, f"enc.{l}.ln2")])
    for l, layer in enumerate(dec.layers):
        _load_attn(layer.self_attn, w, f"dec.{l}.self")
        _load_attn(layer.multihead_attn, w, f"dec.{l}.cross")
        _load_ffn_ln(layer, w, f"dec.{l}.ffn", [(layer.norm1, f"dec.{l}.ln1"), (layer.norm2, f"dec.{l}.ln2"),
                                                 (layer.norm3, f"dec.{l}.ln3")])
    return enc.eval(), dec.eval()


@pytest.mark.parametrize("name,std", [("micro", 0.02), ("micro", 0.3), ("tiny", 0.05)])
def test_encoder_decoder_match_stock_library_transformer(name, std):
    """The post-LN/ReLU encoder and decoder stacks, causal and bidirectional, equal
    torch.nn's Transformer layers loaded with the same weights (float64).  std 0.3
    makes attention far from uniform so that a mask or head-slicing slip shows."""
    dims, w, m = make(name, seed=5, std=std)
    for key in w:  # give biases and LN parameters a visible size as well
        if w[key].ndim == 1 and not key.endswith(".g"):
            w[key] = (w[key] * 10).astype(np.float32)
    m = O.Model(dims, w, np.float64, max_pos=64)
    enc, dec = _torch_stacks(dims, w)
    rng = np.random.default_rng(9)
    src = rng.integers(5, dims["vocab"], size=11)
    tgt = rng.integers(0, dims["vocab"], size=9)
    with torch.no_grad():
        xs = torch.from_numpy(m.embed(src, np.arange(len(src))))[None]
        mem_t = enc(xs)
        memory = m.encode(src)
        assert np.allclose(memory, mem_t[0].numpy(), atol=1e-10)
        xt = torch.from_numpy(m.embed(tgt, np.arange(len(tgt))))[None]
        T = len(tgt)
        causal = torch.triu(torch.full((T, T), float("-inf"), dtype=torch.float64), diagonal=1)
        wout = torch.from_numpy(w["out.w"].astype(np.float64))
        ref_causal = (dec(xt, mem_t, tgt_mask=causal)[0] @ wout.T).numpy()
        ref_bidir = (dec(xt, mem_t)[0] @ wout.T).numpy()
    got_causal = m.decode_full(memory, tgt, causal=True)
    got_bidir = m.decode_full(memory, tgt, causal=False)
    assert np.allclose(got_causal, ref_causal, atol=1e-9)
    assert np.allclose(got_bidir, ref_bidir, atol=1e-9)
    assert np.abs(ref_causal - ref_bidir).max() > 1e-6  # the mask matters in this case


def test_contract_mode_requires_float64_and_stays_close():
    dims = model_dims("micro")
    w = init_weights(dims, 4)
    with pytest.raises(ValueError):
        O.Model(dims, w, np.float32, contract=True)
    exact = O.Model(dims, {k: (O.bf16_round(v) if v.ndim == 2 else v) for k, v in w.items()}, np.float64, max_pos=64)
    con = O.Model(dims, w, np.float64, contract=True, max_pos=64)
    rng = np.random.default_rng(5)
    src = rng.integers(5, dims["vocab"], size=9)
    tgt = rng.integers(0, dims["vocab"], size=7)
    a = exact.decode_full(exact.encode(src), tgt)
    b = con.decode_full(con.encode(src), tgt)
    # bf16 rounding of activations moves logits, but only at the bf16 level
    assert 0 < np.abs(a - b).max() < 2e-2
