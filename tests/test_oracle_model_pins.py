"""Pins of the oracle's model forward against things other than itself.

* the whole decoder against the `transformers` Qwen2 implementation (a library
  routine: the paper's target models are Qwen2-family decoders, Sec. 3/5);
* closed forms for the element-wise pieces;
* KV-cache consistency and the no-speculation identities.
"""
import numpy as np
import pytest
import torch

import das_inputs as di
import oracle


def _hf_model(shape, w):
    from transformers import Qwen2Config, Qwen2ForCausalLM
    cfg = Qwen2Config(vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
                      num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_q_heads,
                      num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                      max_position_embeddings=4096, rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_theta,
                      tie_word_embeddings=False, attention_dropout=0.0, use_sliding_window=False,
                      attn_implementation="eager")
    try:
        cfg.rope_parameters = {"rope_type": "default", "rope_theta": shape.rope_theta}
    except Exception:
        pass
    model = Qwen2ForCausalLM(cfg).to(torch.float64).eval()
    d, qd, kd, F, V = shape.d_model, shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim, shape.d_ffn, shape.vocab
    p = [0]

    def take(*dims):
        n = int(np.prod(dims))
        t = torch.from_numpy(w[p[0]:p[0] + n].astype(np.float64)).reshape(*dims)
        p[0] += n
        return t
    sd = {}
    sd["model.embed_tokens.weight"] = take(V, d)
    for l in range(shape.n_layers):
        pre = f"model.layers.{l}."
        sd[pre + "input_layernorm.weight"] = take(d)
        sd[pre + "self_attn.q_proj.weight"] = take(qd, d)
        sd[pre + "self_attn.k_proj.weight"] = take(kd, d)
        sd[pre + "self_attn.v_proj.weight"] = take(kd, d)
        sd[pre + "self_attn.o_proj.weight"] = take(d, qd)
        sd[pre + "post_attention_layernorm.weight"] = take(d)
        sd[pre + "mlp.gate_proj.weight"] = take(F, d)
        sd[pre + "mlp.up_proj.weight"] = take(F, d)
        sd[pre + "mlp.down_proj.weight"] = take(d, F)
        for nm, n in (("q", qd), ("k", kd), ("v", kd)):
            sd[pre + f"self_attn.{nm}_proj.bias"] = torch.zeros(n, dtype=torch.float64)
    sd["model.norm.weight"] = take(d)
    sd["lm_head.weight"] = take(V, d)
    assert p[0] == w.size
    missing, unexpected = model.load_state_dict(sd, strict=False)
    assert not unexpected, unexpected
    assert all("rotary" in m or "inv_freq" in m for m in missing), missing
    # the library must really be using the theta we asked for
    inv = model.model.rotary_emb.inv_freq.double().numpy()
    want = shape.rope_theta ** (-np.arange(0, shape.head_dim, 2) / shape.head_dim)
    np.testing.assert_allclose(inv, want, rtol=1e-6)
    return model


SHAPES = [
    di.ModelShape("pinA", 2, 64, 4, 2, 16, 96, 50, rope_theta=1.0e4),
    di.ModelShape("pinB", 3, 48, 6, 2, 8, 80, 37, rope_theta=1.0e6, rms_eps=1e-5),
    di.ModelShape("pinC", 1, 32, 2, 2, 16, 40, 20, rope_theta=100.0),     # G = 1
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
def test_forward_matches_transformers_qwen2(shape):
    """All rows' logits of a random model (random gains, sigma large enough that
    attention is far from uniform) equal the library's full-sequence forward."""
    w = di.bf16_to_f32(di.weights_bf16(shape, seed=7, sigma=0.35, gain_sigma=0.2))
    hf = _hf_model(shape, w)
    om = oracle.OracleModel(shape, w)
    rng = np.random.default_rng(3)
    toks = rng.integers(0, shape.vocab, size=23, dtype=np.int32)
    with torch.no_grad():
        ref = hf(torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    s = om.new_seq(64)
    got = om.forward(s, 0, toks)
    assert np.abs(ref).max() > 0.5
    np.testing.assert_allclose(got, ref, rtol=0, atol=2e-5 * max(1.0, np.abs(ref).max()))
    # and block-wise with the KV cache: 10 rows, then 1, then 12
    s2 = om.new_seq(64)
    a = om.forward(s2, 0, toks[:10])
    b = om.forward(s2, 10, toks[10:11])
    c = om.forward(s2, 11, toks[11:])
    np.testing.assert_allclose(np.concatenate([a, b, c]), ref, rtol=0, atol=2e-5 * max(1.0, np.abs(ref).max()))


def test_greedy_decoding_matches_transformers_generate():
    shape = SHAPES[0]
    w = di.bf16_to_f32(di.weights_bf16(shape, seed=11, sigma=0.35, gain_sigma=0.1))
    hf = _hf_model(shape, w)
    om = oracle.OracleModel(shape, w)
    prompt = np.random.default_rng(5).integers(0, shape.vocab, size=9, dtype=np.int32)
    with torch.no_grad():
        out = hf.generate(torch.from_numpy(prompt.astype(np.int64))[None], max_new_tokens=12, do_sample=False,
                          pad_token_id=0, eos_token_id=None)[0].numpy()[len(prompt):]
    s = om.new_seq(64)
    s.pending = int(np.argmax(om.prefill(s, prompt)))
    mine = [s.pending] + om.ar_greedy(s, 11)
    assert mine == [int(t) for t in out]


def test_rmsnorm_closed_forms():
    lib = oracle.model._load()
    d = 64
    g = np.linspace(0.5, 1.5, d).astype(np.float32)
    y = np.empty(d, np.float32)
    x = np.full(d, 3.0, np.float32)
    lib.orc_op_rmsnorm(x.ctypes.data, g.ctypes.data, 1e-6, d, y.ctypes.data)
    np.testing.assert_allclose(y, 3.0 / np.sqrt(9.0 + 1e-6) * g, rtol=1e-6)
    # one-hot: mean square = a^2/d
    x = np.zeros(d, np.float32); x[5] = -2.0
    lib.orc_op_rmsnorm(x.ctypes.data, g.ctypes.data, 1e-6, d, y.ctypes.data)
    assert y[5] == pytest.approx(-2.0 / np.sqrt(4.0 / d + 1e-6) * g[5], rel=1e-6)
    assert np.count_nonzero(y) == 1
    # library routine
    x = np.random.default_rng(0).standard_normal(d).astype(np.float32)
    lib.orc_op_rmsnorm(x.ctypes.data, g.ctypes.data, 1e-5, d, y.ctypes.data)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x).double(), (d,), torch.from_numpy(g).double(), 1e-5)
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-6)


def _rope(x, D, pos, theta):
    lib = oracle.model._load()
    y = np.array(x, dtype=np.float32)
    lib.orc_op_rope(y.ctypes.data, D, pos, theta)
    return y


def test_rope_properties():
    D, theta = 32, 1.0e4
    rng = np.random.default_rng(1)
    q, k = rng.standard_normal(D).astype(np.float32), rng.standard_normal(D).astype(np.float32)
    np.testing.assert_array_equal(_rope(q, D, 0, theta), q)                       # identity at position 0
    assert np.linalg.norm(_rope(q, D, 977, theta)) == pytest.approx(np.linalg.norm(q), rel=1e-6)
    # <R_m q, R_n k> depends on m-n only
    a = float(_rope(q, D, 40, theta) @ _rope(k, D, 33, theta))
    b = float(_rope(q, D, 1007, theta) @ _rope(k, D, 1000, theta))
    c = float(_rope(q, D, 7, theta) @ k)
    assert a == pytest.approx(b, abs=1e-4) and a == pytest.approx(c, abs=1e-4)
    # the pair (i, i+D/2) turns by pos * theta^(-2i/D): unit vector e_0 at pos p -> (cos p, sin p)
    e = np.zeros(D, np.float32); e[0] = 1.0
    r = _rope(e, D, 3, theta)
    assert r[0] == pytest.approx(np.cos(3.0), abs=1e-6) and r[D // 2] == pytest.approx(np.sin(3.0), abs=1e-6)
    e = np.zeros(D, np.float32); e[1] = 1.0
    r = _rope(e, D, 5, theta)
    ang = 5.0 * theta ** (-2.0 / D)
    assert r[1] == pytest.approx(np.cos(ang), abs=1e-6) and r[1 + D // 2] == pytest.approx(np.sin(ang), abs=1e-6)


def test_linear_is_x_times_w_transposed():
    lib = oracle.model._load()
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 70)).astype(np.float32)
    W = rng.standard_normal((33, 70)).astype(np.float32)
    y = np.ones((5, 33), np.float32)
    lib.orc_op_linear(x.ctypes.data, W.ctypes.data, 5, 70, 33, y.ctypes.data, 0)
    np.testing.assert_allclose(y, x.astype(np.float64) @ W.astype(np.float64).T, rtol=1e-6, atol=1e-6)
    lib.orc_op_linear(x.ctypes.data, W.ctypes.data, 5, 70, 33, y.ctypes.data, 1)
    np.testing.assert_allclose(y, 2 * (x.astype(np.float64) @ W.astype(np.float64).T), rtol=1e-5, atol=1e-5)


def test_zero_layers_reduce_to_norm_and_head(tiny_shape):
    """With every per-layer matrix zero the residual stream is the embedding, so
    logits = RMSNorm(E[tok]; gf) Wlm^T (silu(0) = 0, zero attention output)."""
    sh = tiny_shape.replace(vocab=97)
    blob = di.weights_bf16(sh, seed=4, gain_sigma=0.1)
    w = di.bf16_to_f32(blob)
    V, d = sh.vocab, sh.d_model
    E, tail = w[:V * d].reshape(V, d).copy(), w[-(V * d + d):].copy()
    w[V * d: w.size - (V * d + d)] = 0.0
    # restore the two per-layer gain vectors' effect is irrelevant: their inputs are multiplied by zero matrices
    gf, Wlm = tail[:d], tail[d:].reshape(V, d)
    om = oracle.OracleModel(sh, w)
    s = om.new_seq(16)
    toks = np.array([3, 96, 0, 41], np.int32)
    got = om.forward(s, 0, toks)
    x = E[toks].astype(np.float64)
    xn = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + sh.rms_eps) * gf
    np.testing.assert_allclose(got, xn @ Wlm.astype(np.float64).T, rtol=1e-5, atol=1e-6)


def test_kv_cache_consistency_and_batch_independence(tiny_oracle, tiny_shape):
    """prefill(n) last row == prefill(n-m) followed by m more rows."""
    om = tiny_oracle
    prompt = di.prompts([37], tiny_shape.vocab, 9)[0]
    s1 = om.new_seq(64)
    full = om.prefill(s1, prompt)
    s2 = om.new_seq(64)
    om.prefill(s2, prompt[:30])
    part = om.forward(s2, 30, prompt[30:])[-1]
    np.testing.assert_allclose(part, full, atol=1e-5)
    # rows written speculatively and then overwritten leave no trace
    s3 = om.new_seq(64)
    om.prefill(s3, prompt[:30])
    om.forward(s3, 30, np.array([1, 2, 3, 4, 5], np.int32))
    again = om.forward(s3, 30, prompt[30:])[-1]
    np.testing.assert_array_equal(again, part)
