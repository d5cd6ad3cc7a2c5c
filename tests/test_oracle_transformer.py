"""Pins for oracle/transformer.py: every check compares against something that
is not the oracle's own formula -- library routines (Hugging Face reference
decoders, torch SDPA, scipy), brute-force loops, or mathematical invariants."""
import math

import numpy as np
import pytest
import torch

from oracle import transformer as T
from paper_2601_19404_amd import synth


def tiny_shape(cfg=synth.TINY):
    return T.Shape(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                   cfg.d_ffn, cfg.vocab, cfg.rope_base, cfg.rms_eps)


@pytest.fixture(scope="module")
def tiny():
    w = synth.perturb_gains(synth.make_weights(synth.TINY, seed=1234))
    # larger weights than N(0, 0.02) so attention is far from uniform
    for lw in w["layers"]:
        lw["wqkv"] = lw["wqkv"] * 8.0
    w["embed"] = w["embed"] * 20.0
    return tiny_shape(), synth.weights_to_numpy(w)


def test_log_softmax_rows_sum_to_one():
    rng = np.random.default_rng(0)
    z = rng.normal(size=(7, 4099)) * 9.0
    lp = T.log_softmax(z)
    assert np.max(np.abs(np.exp(lp).sum(-1) - 1.0)) < 1e-12


def test_log_softmax_matches_scipy_and_naive():
    from scipy.special import log_softmax
    rng = np.random.default_rng(1)
    z = rng.normal(size=(5, 513))
    np.testing.assert_allclose(T.log_softmax(z), log_softmax(z, axis=-1), atol=1e-13)
    naive = z - np.log(np.exp(z).sum(-1, keepdims=True))
    np.testing.assert_allclose(T.log_softmax(z), naive, atol=1e-13)
    # shift invariance and no overflow at large magnitude
    np.testing.assert_allclose(T.log_softmax(z + 1000.0), T.log_softmax(z), atol=1e-10)


def test_rmsnorm_matches_torch():
    rng = np.random.default_rng(2)
    x = rng.normal(size=(6, 128))
    g = rng.normal(size=128)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (128,), torch.from_numpy(g), 1e-6)
    np.testing.assert_allclose(T.rmsnorm(x, g, 1e-6), ref.numpy(), atol=1e-13)
    # unit gain, eps 0: output rows have unit mean square
    y = T.rmsnorm(x, np.ones(128), 0.0)
    np.testing.assert_allclose((y * y).mean(-1), 1.0, atol=1e-13)


def test_silu_matches_torch():
    x = np.linspace(-20, 20, 401)
    np.testing.assert_allclose(T.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(),
                               atol=1e-14)


def test_rope_position_zero_is_identity_and_norm_preserved():
    rng = np.random.default_rng(3)
    x = rng.normal(size=(5, 3, 32))
    np.testing.assert_array_equal(T.rope(x[:1], np.array([0]), 1e4), x[:1])
    y = T.rope(x, np.arange(5) * 37, 1e4)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), atol=1e-12)


def test_rope_hand_values():
    # dh = 2: a single pair (0, 1) with theta = base^0 = 1: plain rotation by pos radians.
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    y = T.rope(x, np.array([2.0, 0.5]), 1e4)
    np.testing.assert_allclose(y[0, 0], [math.cos(2.0), math.sin(2.0)], atol=1e-15)
    np.testing.assert_allclose(y[1, 0], [-math.sin(0.5), math.cos(0.5)], atol=1e-15)
    # dh = 4: pairs are (0, 2) and (1, 3); second pair turns at base^(-2/4).
    x = np.array([[[1.0, 1.0, 0.0, 0.0]]])
    y = T.rope(x, np.array([3.0]), 100.0)
    th1 = 3.0 * 100.0 ** (-0.5)
    np.testing.assert_allclose(y[0, 0], [math.cos(3.0), math.cos(th1), math.sin(3.0), math.sin(th1)],
                               atol=1e-15)


def test_rope_relative_position_property():
    rng = np.random.default_rng(4)
    q = rng.normal(size=(1, 1, 32))
    k = rng.normal(size=(1, 1, 32))
    def dot(t, u):
        return float(np.sum(T.rope(q, np.array([t]), 1e4) * T.rope(k, np.array([u]), 1e4)))
    assert abs(dot(10, 3) - dot(107, 100)) < 1e-10
    assert abs(dot(10, 3) - dot(7, 0)) < 1e-10
    assert abs(dot(10, 3) - dot(3, 10)) > 1e-3      # not symmetric: sign of rotation matters


def test_attention_matches_torch_sdpa_and_bruteforce():
    shape = T.Shape(1, 64, 4, 2, 16, 8, 8)
    rng = np.random.default_rng(5)
    t = 9
    q = rng.normal(size=(t, 4, 16))
    k = rng.normal(size=(t, 2, 16))
    v = rng.normal(size=(t, 2, 16))
    mask = np.tril(np.ones((t, t), bool))
    out = T.attention_rows(shape, q, k, v, mask)
    # library: SDPA with KV heads replicated (GQA reduces to MHA)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, 2, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, 2, axis=1)).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    np.testing.assert_allclose(out, ref[0].permute(1, 0, 2).numpy(), atol=1e-12)
    # brute force, scalar loops
    for h in range(4):
        for i in range(t):
            sc = [sum(q[i, h, d] * k[u, h // 2, d] for d in range(16)) / 4.0 for u in range(i + 1)]
            mx = max(sc)
            e = [math.exp(s - mx) for s in sc]
            z = sum(e)
            for d in range(16):
                val = sum(e[u] / z * v[u, h // 2, d] for u in range(i + 1))
                assert abs(val - out[i, h, d]) < 1e-12


def _hf_reference(cfg, w_np, kind):
    import transformers
    common = dict(vocab_size=cfg.vocab, hidden_size=cfg.d_model, intermediate_size=cfg.d_ffn,
                  num_hidden_layers=cfg.n_layers, num_attention_heads=cfg.n_q_heads,
                  num_key_value_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                  max_position_embeddings=4096, rms_norm_eps=cfg.rms_eps,
                  rope_theta=cfg.rope_base, tie_word_embeddings=False, hidden_act="silu",
                  attn_implementation="eager")
    if kind == "qwen2":
        model = transformers.Qwen2ForCausalLM(transformers.Qwen2Config(**common))
    else:
        model = transformers.LlamaForCausalLM(transformers.LlamaConfig(
            attention_bias=False, mlp_bias=False, **common))
    model = model.double().eval()
    sd = model.state_dict()
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    nq = cfg.n_q_heads * cfg.head_dim
    nk = cfg.n_kv_heads * cfg.head_dim
    new = {"model.embed_tokens.weight": t(w_np["embed"]), "lm_head.weight": t(w_np["lm_head"]),
           "model.norm.weight": t(w_np["final_norm"])}
    for l, lw in enumerate(w_np["layers"]):
        p = f"model.layers.{l}."
        new[p + "input_layernorm.weight"] = t(lw["attn_norm"])
        new[p + "post_attention_layernorm.weight"] = t(lw["ffn_norm"])
        new[p + "self_attn.q_proj.weight"] = t(lw["wqkv"][:nq])
        new[p + "self_attn.k_proj.weight"] = t(lw["wqkv"][nq:nq + nk])
        new[p + "self_attn.v_proj.weight"] = t(lw["wqkv"][nq + nk:])
        new[p + "self_attn.o_proj.weight"] = t(lw["wo"])
        new[p + "mlp.gate_proj.weight"] = t(lw["w_gate_up"][:cfg.d_ffn])
        new[p + "mlp.up_proj.weight"] = t(lw["w_gate_up"][cfg.d_ffn:])
        new[p + "mlp.down_proj.weight"] = t(lw["w_down"])
    for k in sd:
        if k.endswith(".bias"):
            new[k] = torch.zeros_like(sd[k])       # Qwen2 carries q/k/v biases; ours has none
    missing = [k for k in sd if k not in new and "rotary" not in k]
    assert not missing, missing
    model.load_state_dict(new, strict=False)
    return model


@pytest.mark.parametrize("kind", ["qwen2", "llama"])
def test_full_forward_matches_huggingface_reference(tiny, kind):
    """The whole decoder (embedding, RMSNorm placement and eps, RoPE pairing and
    base, GQA head mapping, 1/sqrt(dh), SwiGLU, untied head) against the public
    reference implementation of the model family the paper trains."""
    shape, w = tiny
    model = _hf_reference(synth.TINY, w, kind)
    rng = np.random.default_rng(6)
    toks = rng.integers(0, shape.vocab, size=40)
    with torch.no_grad():
        ref = model(torch.from_numpy(toks)[None]).logits[0].numpy()
    got = T.logits_full(shape, w, toks)
    assert ref.std() > 0.1
    # The reference module evaluates its rotary angles in fp32 even when the model
    # is cast to fp64, which leaves ~4e-7 of noise; a structural mistake (pairing,
    # head mapping, norm placement, scale) moves logits by >1e-2.
    np.testing.assert_allclose(got, ref, atol=5e-6)


def test_incremental_equals_full(tiny):
    shape, w = tiny
    rng = np.random.default_rng(7)
    toks = rng.integers(0, shape.vocab, size=30)
    full = T.logits_full(shape, w, toks)
    kv, z_last = T.prefill(shape, w, toks[:21])
    np.testing.assert_allclose(z_last, full[20], atol=1e-10)
    for j in range(21, 30):
        z = T.decode_step(shape, w, int(toks[j]), kv)
        np.testing.assert_allclose(z, full[j], atol=1e-10)
    # chunked prefill (two chunks) as well
    kv2 = T.KV(shape)
    T.hidden_incremental(shape, w, toks[:13], kv2)
    h = T.hidden_incremental(shape, w, toks[13:30], kv2)
    np.testing.assert_allclose(T.lm_head(w, h), full[13:30], atol=1e-10)


def test_causality_future_tokens_do_not_matter(tiny):
    shape, w = tiny
    rng = np.random.default_rng(8)
    toks = rng.integers(0, shape.vocab, size=24)
    a = T.logits_full(shape, w, toks)
    toks2 = toks.copy()
    toks2[15:] = rng.integers(0, shape.vocab, size=9)
    b = T.logits_full(shape, w, toks2)
    np.testing.assert_array_equal(a[:15], b[:15])
    assert np.max(np.abs(a[15:] - b[15:])) > 1e-3


def test_gqa_reduces_to_mha_when_kv_heads_replicated(tiny):
    shape, w = tiny
    per = shape.n_q_heads // shape.n_kv_heads
    dh = shape.head_dim
    nq, nk = shape.n_q_heads * dh, shape.n_kv_heads * dh
    w2 = dict(w, layers=[])
    for lw in w["layers"]:
        wq, wk, wv = lw["wqkv"][:nq], lw["wqkv"][nq:nq + nk], lw["wqkv"][nq + nk:]
        rep = lambda a: np.repeat(a.reshape(shape.n_kv_heads, dh, -1), per, axis=0).reshape(nq, -1)
        w2["layers"].append(dict(lw, wqkv=np.concatenate([wq, rep(wk), rep(wv)])))
    shape2 = T.Shape(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_q_heads, dh,
                     shape.d_ffn, shape.vocab, shape.rope_base, shape.rms_eps)
    toks = np.random.default_rng(9).integers(0, shape.vocab, size=17)
    np.testing.assert_allclose(T.logits_full(shape2, w2, toks), T.logits_full(shape, w, toks),
                               atol=1e-10)


def test_teacher_forced_rows_and_suffix_logprobs(tiny):
    shape, w = tiny
    rng = np.random.default_rng(10)
    prefix = rng.integers(0, shape.vocab, size=19)
    suffix = rng.integers(0, shape.vocab, size=7)
    rows = T.teacher_forced_logits(shape, w, prefix, suffix)
    full = T.logits_full(shape, w, np.concatenate([prefix, suffix]))
    np.testing.assert_allclose(rows, full[18:25], atol=1e-10)   # row S-1 scores the first suffix token
    for temp in (1.0, 0.7):
        lp = T.suffix_logprobs(shape, w, prefix, suffix, temp)
        ref = torch.log_softmax(torch.from_numpy(full[18:25]) / temp, -1).numpy()[np.arange(7), suffix]
        np.testing.assert_allclose(lp, ref, atol=1e-10)
    assert T.suffix_logprobs(shape, w, prefix, suffix[:0]).shape == (0,)


def test_round_bf16_matches_library_and_hand_values():
    rng = np.random.default_rng(11)
    x = np.concatenate([rng.normal(size=5000) * 10.0 ** rng.integers(-6, 6, size=5000),
                        [0.0, -0.0, 1.0, -1.0, 3.0e38, 1e-40]])
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(T.round_bf16(x), ref)
    # ties go to the even significand; anything above the tie goes up
    assert T.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert T.round_bf16(np.array([1.0 + 2.0 ** -7 + 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert T.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1.0 + 2.0 ** -7
    y = T.round_bf16(x)
    np.testing.assert_array_equal(T.round_bf16(y), y)            # idempotent
    assert np.isnan(T.round_bf16(np.array([np.nan]))[0]) and np.isinf(T.round_bf16(np.array([np.inf]))[0])


def test_bf16_storage_mode_is_a_small_perturbation_and_consistent(tiny):
    """Quantising the stored tensors moves the logits by about 2^-9 relative (not more: a
    misplaced rounding of an accumulator would), and the two evaluation orders still agree
    exactly enough (same values are rounded in both)."""
    shape, w = tiny
    sb = T.Shape(**{**shape.__dict__, "storage": "bf16"})
    toks = np.random.default_rng(12).integers(0, shape.vocab, size=24)
    exact = T.logits_full(shape, w, toks)
    quant = T.logits_full(sb, w, toks)
    err = np.abs(quant - exact).max() / exact.std()
    assert 1e-4 < err < 5e-2
    kv, z = T.prefill(sb, w, toks[:17])
    np.testing.assert_allclose(z, quant[16], atol=1e-9)
    for j in range(17, 24):
        np.testing.assert_allclose(T.decode_step(sb, w, int(toks[j]), kv), quant[j], atol=1e-9)
