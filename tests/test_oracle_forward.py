"""Pins for the oracle's transformer forward and top-1 confidence (CPU only).

The forward is pinned against things other than itself: third-party library routines that
implement the same layers (torch SDPA / rms_norm / silu, and whole HF Llama / Qwen2 stacks
run with an all-visible attention mask), structural special cases (zeroed output
projections, one-token sequences, uniform values), and symmetries a bidirectional model
must have (permutation equivariance without rotary phases; rotary scores depend only on
relative position).  The confidence is pinned by closed forms (Sec. 3.1: c = max_v p).
"""
import dataclasses

import numpy as np
import pytest
import torch

import psd_inputs as inp
from oracle import psd_oracle as orc

TINY = inp.WORKLOADS[1].shape
GQA = inp.cut_down(inp.WORKLOADS[4].shape, name="gqa-tiny", dtype="fp32", n_layers=2, d_model=96, n_heads=6,
                   n_kv_heads=2, d_head=16, d_ffn=160, vocab=211, seed=11)


def _tokens(shape, N, seed, frac_mask=0.4):
    rng = np.random.default_rng(seed)
    t = rng.integers(0, shape.vocab - 1, size=N).astype(np.int32)
    t[rng.random(N) < frac_mask] = shape.mask_id
    return t


# ---------------------------------------------------------------- library-routine pins


def test_rmsnorm_silu_match_torch_functional():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((7, 48))
    g = rng.standard_normal(48)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), eps=1e-5).numpy()
    np.testing.assert_allclose(orc.rmsnorm(x, g, 1e-5), ref, rtol=0, atol=1e-13)
    np.testing.assert_allclose(orc.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(), atol=1e-14)


@pytest.mark.parametrize("H,Hkv", [(4, 4), (6, 2), (8, 1)])
def test_attention_matches_torch_sdpa(H, Hkv):
    rng = np.random.default_rng(H * 10 + Hkv)
    N, dh = 13, 16
    q = rng.standard_normal((N, H, dh))
    k = rng.standard_normal((N, Hkv, dh))
    v = rng.standard_normal((N, Hkv, dh))
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=False, enable_gqa=True)
    np.testing.assert_allclose(orc.attention(q, k, v), ref[0].permute(1, 0, 2).numpy(), atol=1e-12)


def _hf_model(shape, model):
    """The same weights loaded into a HuggingFace stack (test-only, third-party routine)."""
    from transformers import LlamaConfig, LlamaModel, Qwen2Config, Qwen2Model
    kw = dict(hidden_size=shape.d_model, intermediate_size=shape.d_ffn, num_hidden_layers=shape.n_layers,
              num_attention_heads=shape.n_heads, num_key_value_heads=shape.n_kv_heads, vocab_size=shape.vocab,
              rms_norm_eps=shape.rms_eps, rope_theta=shape.rope_theta, max_position_embeddings=model.max_seq)
    if shape.qkv_bias:
        cfg = Qwen2Config(**kw)
        cfg._attn_implementation = "eager"
        hf = Qwen2Model(cfg)
    else:
        cfg = LlamaConfig(attention_bias=False, **kw)
        cfg._attn_implementation = "eager"
        hf = LlamaModel(cfg)
    hf = hf.double().eval()
    sd = {"embed_tokens.weight": model.tok_emb, "norm.weight": model.final_norm}
    names = {"attn_norm": "input_layernorm.weight", "ffn_norm": "post_attention_layernorm.weight",
             "wq": "self_attn.q_proj.weight", "wk": "self_attn.k_proj.weight", "wv": "self_attn.v_proj.weight",
             "bq": "self_attn.q_proj.bias", "bk": "self_attn.k_proj.bias", "bv": "self_attn.v_proj.bias",
             "wo": "self_attn.o_proj.weight", "w_gate": "mlp.gate_proj.weight", "w_up": "mlp.up_proj.weight",
             "w_down": "mlp.down_proj.weight"}
    for l, lw in enumerate(model.layers):
        for k, v in lw.items():
            if v is not None:
                sd[f"layers.{l}.{names[k]}"] = v
    missing, unexpected = hf.load_state_dict({k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in sd.items()},
                                             strict=False)
    assert not unexpected and all("rotary" in m or "inv_freq" in m for m in missing), (missing, unexpected)
    return hf


@pytest.mark.parametrize("shape", [TINY, GQA], ids=["mha-nobias", "gqa-bias"])
def test_forward_matches_hf_stack_with_all_visible_mask(shape):
    N = 24
    model = inp.draw_model(shape, max_seq=N)
    # non-trivial norm gains so that a dropped gain would show
    rng = np.random.default_rng(5)
    model.final_norm = (1 + 0.3 * rng.standard_normal(shape.d_model)).astype(np.float32)
    for lw in model.layers:
        lw["attn_norm"] = (1 + 0.3 * rng.standard_normal(shape.d_model)).astype(np.float32)
        lw["ffn_norm"] = (1 + 0.3 * rng.standard_normal(shape.d_model)).astype(np.float32)
        for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            lw[k] = lw[k] * np.float32(12.0)       # make attention and FFN matter at this width
    tokens = _tokens(shape, N, 3)
    hf = _hf_model(shape, model)
    with torch.no_grad():
        ref = hf(input_ids=torch.from_numpy(tokens.astype(np.int64))[None],
                 attention_mask=torch.zeros(1, 1, N, N, dtype=torch.float64)).last_hidden_state[0].numpy()
    y = orc.forward_hidden(model, tokens)
    assert np.abs(ref).max() > 0.5
    np.testing.assert_allclose(y, ref, atol=2e-5, rtol=0)       # fp32 rotary tables on both sides
    # and the pin has teeth: a causal run of the same stack differs
    with torch.no_grad():
        causal = hf(input_ids=torch.from_numpy(tokens.astype(np.int64))[None]).last_hidden_state[0].numpy()
    assert np.abs(causal - y).max() > 1e-3


# ---------------------------------------------------------------- structural special cases


def test_zero_output_projections_leave_residual_untouched():
    model = inp.draw_model(TINY, max_seq=16)
    for lw in model.layers:
        lw["wo"] = np.zeros_like(lw["wo"])
        lw["w_down"] = np.zeros_like(lw["w_down"])
    tokens = _tokens(TINY, 16, 0)
    e = model.tok_emb[tokens].astype(np.float64)
    expect = e / np.sqrt((e * e).mean(-1, keepdims=True) + TINY.rms_eps)
    np.testing.assert_allclose(orc.forward_hidden(model, tokens), expect, atol=1e-14)


def test_single_token_attention_is_identity_on_values():
    rng = np.random.default_rng(2)
    q, k, v = (rng.standard_normal((1, 4, 16)) for _ in range(3))
    np.testing.assert_allclose(orc.attention(q, k, v), v, atol=1e-15)


def test_uniform_values_pass_through_attention():
    rng = np.random.default_rng(3)
    q, k = rng.standard_normal((9, 4, 16)), rng.standard_normal((9, 2, 16))
    v = np.tile(rng.standard_normal((1, 2, 16)), (9, 1, 1))
    out = orc.attention(q, k, v)
    np.testing.assert_allclose(out, np.repeat(v, 2, axis=1), atol=1e-14)


def test_attention_weights_follow_softmax_of_scaled_scores():
    # two keys, one query: output = v0 + sigmoid((q.k1 - q.k0)/sqrt(dh)) (v1 - v0)
    rng = np.random.default_rng(4)
    dh = 8
    q = rng.standard_normal((2, 1, dh))
    k = rng.standard_normal((2, 1, dh))
    v = rng.standard_normal((2, 1, dh))
    out = orc.attention(q, k, v)
    for i in range(2):
        w1 = 1 / (1 + np.exp(-(q[i, 0] @ (k[1, 0] - k[0, 0])) / np.sqrt(dh)))
        np.testing.assert_allclose(out[i, 0], v[0, 0] + w1 * (v[1, 0] - v[0, 0]), atol=1e-14)


def test_bidirectional_model_is_permutation_equivariant_without_rotary_phase():
    N = 12
    model = inp.draw_model(GQA, max_seq=N)
    model.rope_cos = np.ones_like(model.rope_cos)
    model.rope_sin = np.zeros_like(model.rope_sin)
    for lw in model.layers:
        for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            lw[k] = lw[k] * np.float32(12.0)
    tokens = _tokens(GQA, N, 7)
    perm = np.random.default_rng(8).permutation(N)
    y = orc.forward_hidden(model, tokens)
    yp = orc.forward_hidden(model, tokens[perm])
    np.testing.assert_allclose(yp, y[perm], atol=1e-12)
    # every position sees every other one (no causal mask): changing the last token moves row 0
    t2 = tokens.copy()
    t2[-1] = (t2[-1] + 1) % (GQA.vocab - 1)
    assert np.abs(orc.forward_hidden(model, t2)[0] - y[0]).max() > 1e-6


def test_rope_is_a_rotation_and_scores_depend_on_relative_position_only():
    shape = dataclasses.replace(TINY, d_head=16)
    cos, sin = (a.astype(np.float64) for a in inp.rope_tables(shape, 64))
    rng = np.random.default_rng(9)
    q = rng.standard_normal((64, 1, 16))
    k = rng.standard_normal((64, 1, 16))
    rq, rk = orc.rope(q, cos, sin), orc.rope(k, cos, sin)
    np.testing.assert_allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-7)
    np.testing.assert_allclose(rq[0], q[0], atol=1e-15)                 # position 0: identity
    # same vectors placed at (i, j) and (i+s, j+s) give the same score
    qq = np.tile(q[:1], (64, 1, 1))
    kk = np.tile(k[:1], (64, 1, 1))
    rqq, rkk = orc.rope(qq, cos, sin), orc.rope(kk, cos, sin)
    s_a = rqq[5, 0] @ rkk[2, 0]
    s_b = rqq[45, 0] @ rkk[42, 0]
    s_c = rqq[2, 0] @ rkk[5, 0]
    np.testing.assert_allclose(s_a, s_b, atol=1e-5)                     # fp32 tables
    assert abs(s_a - s_c) > 1e-3                                        # sign of the offset matters
    # pairing is (j, j + d_head/2) with angle pos * theta^(-2j/d_head): check one pair by hand
    pos, j = 7, 3
    ang = pos * shape.rope_theta ** (-2.0 * j / 16)
    x1, x2 = q[pos, 0, j], q[pos, 0, j + 8]
    np.testing.assert_allclose(rq[pos, 0, j], x1 * np.cos(ang) - x2 * np.sin(ang), atol=1e-6)
    np.testing.assert_allclose(rq[pos, 0, j + 8], x2 * np.cos(ang) + x1 * np.sin(ang), atol=1e-6)


# ---------------------------------------------------------------- confidence closed forms


def test_confidence_closed_forms():
    V, mask_id = 50, 49
    z = np.full((1, V), 0.7)
    x_hat, c = orc.top1_confidence(z, mask_id)
    assert x_hat[0] == 0 and c[0] == pytest.approx(1.0 / (V - 1), rel=1e-14)
    for delta in (0.5, 3.0, 12.0):
        z = np.full((1, V), -1.3)
        z[0, 17] += delta
        x_hat, c = orc.top1_confidence(z, mask_id)
        assert x_hat[0] == 17
        assert c[0] == pytest.approx(1.0 / (1.0 + (V - 2) * np.exp(-delta)), rel=1e-13)


def test_mask_token_is_never_predicted_and_not_in_the_normaliser():
    V, mask_id = 20, 19
    z = np.zeros((2, V))
    z[:, mask_id] = 50.0           # would dominate if it were part of the vocabulary
    z[1, 4] = 1.0
    x_hat, c = orc.top1_confidence(z, mask_id)
    assert list(x_hat) == [0, 4]
    assert c[0] == pytest.approx(1 / 19)
    assert c[1] == pytest.approx(np.e / (np.e + 18))


def test_confidence_equals_max_of_library_softmax_and_ties_go_low():
    from scipy.special import softmax
    rng = np.random.default_rng(10)
    V, mask_id = 300, 299
    z = rng.standard_normal((40, V)) * 3
    z[5, 100] = z[5, 200] = z[5].max() + 1.0         # exact tie
    x_hat, c = orc.top1_confidence(z, mask_id)
    p = softmax(z[:, :mask_id], axis=-1)
    np.testing.assert_array_equal(x_hat, p.argmax(-1))
    np.testing.assert_allclose(c, p.max(-1), rtol=1e-12)
    assert x_hat[5] == 100


def test_forward_confidence_sentinels_and_logit_scale():
    shape = TINY
    model = inp.draw_model(shape, max_seq=48)
    w = inp.WORKLOADS[1]
    tokens = inp.initial_state(w)[0]
    tokens[20] = 5                                  # one committed position inside the block
    top1, conf, z = orc.forward_confidence(model, tokens, 16, 32, return_logits=True)
    assert top1[4] == 5 and conf[4] == -1.0
    live = np.arange(32) != 4
    assert (conf[live] > 1.0 / shape.vocab).all() and (conf[live] < 1).all() and (top1[live] != shape.mask_id).all()
    # logits are y W^T with y the final-normed hidden state: check one entry from its definition
    y = orc.forward_hidden(model, tokens)
    assert z[7, 33] == pytest.approx(float(y[16 + 7] @ model.lm_head[33].astype(np.float64)), rel=1e-12)
    # a sharper head (logit_scale) raises every top-1 confidence, and leaves the argmax alone
    model2 = dataclasses.replace(model, shape=dataclasses.replace(shape, logit_scale=4.0))
    top1b, confb = orc.forward_confidence(model2, tokens, 16, 32)
    assert (top1b == top1).all() and (confb[live] > conf[live]).all()


# ---------------------------------------------------------------- bf16-operand evaluation


def test_to_bf16_is_the_library_rounding_including_ties():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(4096) * 10.0 ** rng.integers(-6, 6, size=4096),
                        # exact halfway cases between neighbouring bf16 values (ties go to the even significand)
                        np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(2.0 + 2.0 ** -7), 0.5 + 2.0 ** -9, 0.0, -0.0])])
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    got = orc.to_bf16(x)
    assert np.array_equal(got, ref)
    assert np.array_equal(orc.to_bf16(got), got)   # idempotent


def _torch_bf16_operand_layer(h, lw, shape, cos, sin):
    """The same layer with torch: every contraction operand cast to bfloat16 by the library, products and sums
    in float64."""
    def op(t):
        return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)

    def w(name):
        return torch.from_numpy(np.asarray(lw[name], dtype=np.float64))

    N, H, Hkv, dh = h.shape[0], shape.n_heads, shape.n_kv_heads, shape.d_head
    tcos, tsin = torch.from_numpy(cos)[:, None, :], torch.from_numpy(sin)[:, None, :]

    def rot(x):
        x1, x2 = x[..., : dh // 2], x[..., dh // 2:]
        return torch.cat([x1 * tcos - x2 * tsin, x2 * tcos + x1 * tsin], dim=-1)

    a = op(torch.nn.functional.rms_norm(h, (h.shape[1],), w("attn_norm"), eps=shape.rms_eps))
    q, k, v = a @ w("wq").T, a @ w("wk").T, a @ w("wv").T
    if lw.get("bq") is not None:
        q, k, v = q + w("bq"), k + w("bk"), v + w("bv")
    q, k, v = op(rot(q.reshape(N, H, dh))), op(rot(k.reshape(N, Hkv, dh))), op(v.reshape(N, Hkv, dh))
    o = torch.empty(N, H, dh, dtype=torch.float64)
    for j in range(H):
        s = q[:, j] @ k[:, j // (H // Hkv)].T / np.sqrt(dh)
        e = torch.exp(s - s.max(dim=-1, keepdim=True).values)
        o[:, j] = (op(e) @ v[:, j // (H // Hkv)]) / e.sum(dim=-1, keepdim=True)
    h = h + op(o.reshape(N, H * dh)) @ w("wo").T
    f = op(torch.nn.functional.rms_norm(h, (h.shape[1],), w("ffn_norm"), eps=shape.rms_eps))
    g = op(torch.nn.functional.silu(f @ w("w_gate").T) * (f @ w("w_up").T))
    return h + g @ w("w_down").T


@pytest.mark.parametrize("shape", [TINY, GQA], ids=["mha", "gqa-bias"])
def test_bf16_operand_layer_rounds_exactly_the_contraction_inputs(shape):
    """operands="bf16": each contraction input goes through the bf16 rounding and nothing else does (checked
    against a torch evaluation that casts the same operands with the library's bfloat16)."""
    N = 11
    model = inp.draw_model(shape, N)
    rng = np.random.default_rng(3)
    h = rng.standard_normal((N, shape.d_model))
    cos, sin = np.asarray(model.rope_cos[:N], dtype=np.float64), np.asarray(model.rope_sin[:N], dtype=np.float64)
    got = orc.layer_forward(h, model.layers[0], shape, cos, sin, operands="bf16")
    ref = _torch_bf16_operand_layer(torch.from_numpy(h), model.layers[0], shape, cos, sin).numpy()
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    exact = orc.layer_forward(h, model.layers[0], shape, cos, sin)
    dev = np.abs(got - exact).max()
    assert 0 < dev < 2e-2 * np.abs(exact).max()   # it does round, and by about 2^-9 relative


def test_bf16_operand_logits_round_the_final_hidden_rows_and_stay_close_to_exact():
    shape = GQA
    N, bs, L = 12, 4, 8
    model = inp.draw_model(shape, N)
    t = _tokens(shape, N, 8)
    y_exact = orc.forward_hidden(model, t)
    y_b = orc.forward_hidden(model, t, operands="bf16")
    assert np.array_equal(orc.to_bf16(y_b), y_b)            # the LM-head operand is bf16
    z, z_b = orc.block_logits(model, t, bs, L), orc.block_logits(model, t, bs, L, operands="bf16")
    np.testing.assert_allclose(z_b, y_b[bs: bs + L] @ np.asarray(model.lm_head, dtype=np.float64).T, atol=1e-12)
    rel = np.abs(z_b - z).max() / np.abs(z).max()
    assert 0 < rel < 0.05 and np.abs(y_b - y_exact).max() < 0.05


# ---------------------------------------------------------------- context-causal block attention (App. A)


def test_block_causal_attention_special_cases_and_library_mask():
    rng = np.random.default_rng(21)
    N, H, Hkv, dh = 24, 4, 2, 16
    q, k, v = rng.standard_normal((N, H, dh)), rng.standard_normal((N, Hkv, dh)), rng.standard_normal((N, Hkv, dh))
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    sdpa = torch.nn.functional.scaled_dot_product_attention
    # blocks of one token: ordinary causal attention
    ref = sdpa(tq, tk, tv, is_causal=True, enable_gqa=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(orc.attention(q, k, v, visible=orc.block_causal_visibility(N, 1)), ref, atol=1e-12)
    # one block covering everything: bidirectional
    np.testing.assert_allclose(orc.attention(q, k, v, visible=orc.block_causal_visibility(N, N)), orc.attention(q, k, v),
                               atol=1e-14)
    # any block length: the library's attention under the mask written out from the definition
    for L in (4, 8, 12):
        vis = np.array([[(j // L) <= (i // L) for j in range(N)] for i in range(N)])
        assert np.array_equal(orc.block_causal_visibility(N, L), vis)
        ref = sdpa(tq, tk, tv, attn_mask=torch.from_numpy(vis), enable_gqa=True)[0].permute(1, 0, 2).numpy()
        np.testing.assert_allclose(orc.attention(q, k, v, visible=vis), ref, atol=1e-12)


@pytest.mark.parametrize("shape", [TINY, GQA], ids=["llama-mha", "qwen2-gqa-bias"])
def test_block_causal_forward_matches_hf_stack_with_the_same_mask(shape):
    N, L = 24, 8
    model = inp.draw_model(shape, N)
    hf = _hf_model(shape, model)
    t = _tokens(shape, N, 17)
    vis = orc.block_causal_visibility(N, L)
    mask = torch.where(torch.from_numpy(vis), 0.0, float("-inf")).to(torch.float32)[None, None]
    with torch.no_grad():
        ref = hf(input_ids=torch.from_numpy(t.astype(np.int64))[None], attention_mask=mask).last_hidden_state[0].numpy()
    np.testing.assert_allclose(orc.forward_hidden(model, t, block_causal=L), ref, rtol=0, atol=2e-5)


def test_block_causal_prefix_is_independent_of_what_follows():
    """What makes a prefix KV cache exact: the hidden states of finished blocks depend on nothing after them,
    and the active block depends on later positions not at all."""
    shape, N, L = GQA, 32, 8
    model = inp.draw_model(shape, N)
    t = _tokens(shape, N, 23)
    y = orc.forward_hidden(model, t, block_causal=L)
    t2 = t.copy()
    t2[2 * L:] = (t2[2 * L:] + 7) % (shape.vocab - 1)            # rewrite blocks 2 and 3
    y2 = orc.forward_hidden(model, t2, block_causal=L)
    np.testing.assert_allclose(y2[: 2 * L], y[: 2 * L], atol=1e-13)
    assert np.abs(y2[2 * L:] - y[2 * L:]).max() > 1e-3
    # truncating the sequence after a block changes nothing before the cut
    np.testing.assert_allclose(orc.forward_hidden(model, t[: 3 * L], block_causal=L), y[: 3 * L], atol=1e-13)
    # and the bidirectional model does not have that property
    assert np.abs(orc.forward_hidden(model, t2)[: 2 * L] - orc.forward_hidden(model, t)[: 2 * L]).max() > 1e-3
    with pytest.raises(ValueError):
        orc.block_logits(model, t, 4, L, block_causal=True)


# ---------------------------------------------------------------- approximate KV cache for bidirectional models


def _torch_stack(model, tokens, override=None, keep_rows=None):
    """The whole layer stack over ALL N rows with torch (float64).  Returns (final-normed hidden states [N, d], list of
    per-layer (rotated keys, values)).  override: per-layer (k, v) whose rows `keep_rows` replace the freshly computed
    ones before the attention -- i.e. those positions' keys and values are frozen."""
    shape = model.shape
    N, H, Hkv, dh = len(tokens), shape.n_heads, shape.n_kv_heads, shape.d_head
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    tcos, tsin = t(model.rope_cos[:N])[:, None, :], t(model.rope_sin[:N])[:, None, :]

    def rot(x):
        x1, x2 = x[..., : dh // 2], x[..., dh // 2:]
        return torch.cat([x1 * tcos - x2 * tsin, x2 * tcos + x1 * tsin], dim=-1)

    h = t(model.tok_emb[np.asarray(tokens)])
    kvs = []
    for li, lw in enumerate(model.layers):
        a = torch.nn.functional.rms_norm(h, (h.shape[1],), t(lw["attn_norm"]), eps=shape.rms_eps)
        q, k, v = a @ t(lw["wq"]).T, a @ t(lw["wk"]).T, a @ t(lw["wv"]).T
        if lw.get("bq") is not None:
            q, k, v = q + t(lw["bq"]), k + t(lw["bk"]), v + t(lw["bv"])
        q, k, v = rot(q.reshape(N, H, dh)), rot(k.reshape(N, Hkv, dh)), v.reshape(N, Hkv, dh)
        if override is not None:
            k, v = k.clone(), v.clone()
            k[keep_rows], v[keep_rows] = override[li][0][keep_rows], override[li][1][keep_rows]
        kvs.append((k, v))
        rep = H // Hkv
        o = torch.nn.functional.scaled_dot_product_attention(q.transpose(0, 1), k.repeat_interleave(rep, 1).transpose(0, 1),
                                                             v.repeat_interleave(rep, 1).transpose(0, 1)).transpose(0, 1)
        h = h + o.reshape(N, H * dh) @ t(lw["wo"]).T
        f = torch.nn.functional.rms_norm(h, (h.shape[1],), t(lw["ffn_norm"]), eps=shape.rms_eps)
        h = h + (torch.nn.functional.silu(f @ t(lw["w_gate"]).T) * (f @ t(lw["w_up"]).T)) @ t(lw["w_down"]).T
    return torch.nn.functional.rms_norm(h, (h.shape[1],), t(model.final_norm), eps=shape.rms_eps), kvs


@pytest.mark.parametrize("shape", [TINY, GQA], ids=["mha", "gqa-bias"])
def test_approximate_cache_first_call_exact_then_block_rows_against_frozen_keys_and_values(shape):
    """The approximate cache is pinned by an independent torch evaluation over all N rows: the first call on a block is
    the exact forward; a later call equals the full stack in which, at every layer, the keys and values of the
    positions outside the block are overwritten by those of the first call (so the block rows see stale context, and
    nothing else differs).  Unchanged block content reproduces the exact forward; changed content does not."""
    N, L, start = 40, 8, 16
    model = inp.draw_model(shape, N)
    t0 = _tokens(shape, N, 5)
    t0[start:start + L] = shape.mask_id
    cache = orc.ApproximateCache(model)
    top1, conf = cache(t0, start, L)
    ex_top1, ex_conf, ex_z = orc.forward_confidence(model, t0, start, L, return_logits=True)
    assert (top1 == ex_top1).all() and (conf == ex_conf).all() and cache.refreshes == 1
    np.testing.assert_allclose(cache.logits, ex_z, rtol=0, atol=1e-12)
    y0, kv0 = _torch_stack(model, t0)
    np.testing.assert_allclose(y0[start:start + L].numpy() @ np.asarray(model.lm_head, dtype=np.float64).T * shape.logit_scale,
                               ex_z, rtol=0, atol=1e-9)
    # same content again: the frozen keys / values are exact, so is the result
    cache(t0, start, L)
    np.testing.assert_allclose(cache.logits, ex_z, rtol=0, atol=1e-10)
    assert cache.refreshes == 1
    # three block positions committed: block rows recomputed, the rest of the sequence frozen
    t1 = t0.copy()
    t1[[start + 1, start + 4, start + 7]] = [3, 9, 27]
    top1, conf = cache(t1, start, L)
    outside = np.r_[0:start, start + L:N]
    y1, _ = _torch_stack(model, t1, override=kv0, keep_rows=torch.from_numpy(outside))
    z_ref = y1[start:start + L].numpy() @ np.asarray(model.lm_head, dtype=np.float64).T * shape.logit_scale
    np.testing.assert_allclose(cache.logits, z_ref, rtol=0, atol=1e-9)
    z_exact = orc.forward_confidence(model, t1, start, L, return_logits=True)[2]
    gap = np.abs(cache.logits - z_exact).max()
    assert 1e-6 < gap < 0.5 * np.abs(z_exact).max()           # an approximation, and a mild one
    assert (top1[[1, 4, 7]] == [3, 9, 27]).all() and (conf[[1, 4, 7]] == -1).all()
    # another block refreshes; tokens changed outside the cached block are refused
    cache(t1, start + L, L)
    assert cache.refreshes == 2
    bad = t1.copy()
    bad[2] = (bad[2] + 1) % (shape.vocab - 1)
    with pytest.raises(ValueError):
        cache(bad, start + L, L)


def test_approximate_cache_is_exact_when_the_block_is_the_whole_sequence_and_decodes_to_completion():
    shape = TINY
    N = 24
    model = inp.draw_model(shape, N)
    t = np.full(N, shape.mask_id, dtype=np.int32)
    cache = orc.ApproximateCache(model)
    cache(t, 0, N)
    t2 = t.copy()
    t2[5] = 17
    cache(t2, 0, N)                                                # nothing outside the block: no stale context
    np.testing.assert_allclose(cache.logits, orc.forward_confidence(model, t2, 0, N, return_logits=True)[2], rtol=0, atol=1e-10)
    # the decode loop runs on it like on any model call: one refresh per block, every token resolved, TPF >= 1
    P, L = 8, 8
    x = np.full(P + 2 * L, shape.mask_id, dtype=np.int32)
    x[:P] = inp.draw_prompt(shape.vocab, P, 3)
    cache = orc.ApproximateCache(model)
    out, st = orc.decode(cache, x, P, L, orc.Policy(0.9, 1), orc.chain_graph(3), shape.mask_id)
    assert not (out == shape.mask_id).any() and cache.refreshes == 2 and st.tokens == 2 * L and st.tpf >= 1.0
