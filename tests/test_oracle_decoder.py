"""Pins for oracle/decoder.py: each test ties a function to something other
than itself (brute force written out with scalar loops, closed forms,
invariances, or the public Qwen2 implementation in the `transformers`
library)."""
import math

import numpy as np
import pytest

from oracle import decoder
from paper_2505_24298_amd import synth


# ---------------------------------------------------------------- attention
def _brute_attention(q, k, v):
    Tq, nq, d = q.shape
    nkv = k.shape[1]
    out = np.zeros_like(q)
    for i in range(Tq):
        for a in range(nq):
            kv = a // (nq // nkv)
            s = [sum(q[i, a, e] * k[j, kv, e] for e in range(d)) / math.sqrt(d)
                 for j in range(i + 1)]
            mx = max(s)
            p = [math.exp(x - mx) for x in s]
            z = sum(p)
            for e in range(d):
                out[i, a, e] = sum(p[j] / z * v[j, kv, e] for j in range(i + 1))
    return out


def test_attention_matches_brute_force():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((7, 4, 6))
    k = rng.standard_normal((7, 2, 6))
    v = rng.standard_normal((7, 2, 6))
    np.testing.assert_allclose(decoder.causal_attention(q, k, v), _brute_attention(q, k, v),
                               rtol=0, atol=1e-12)


def test_softmax_rows_sum_to_one():
    rng = np.random.default_rng(2)
    p = decoder.softmax_rows(rng.standard_normal((50, 33)) * 10)
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-12)
    assert (p >= 0).all()


def test_attention_equal_keys_gives_running_mean():
    rng = np.random.default_rng(3)
    T = 9
    q = rng.standard_normal((T, 2, 4))
    k = np.tile(rng.standard_normal((1, 1, 4)), (T, 1, 1))
    v = rng.standard_normal((T, 1, 4))
    o = decoder.causal_attention(q, k, v)
    mean = np.cumsum(v[:, 0, :], axis=0) / np.arange(1, T + 1)[:, None]
    for a in range(2):
        np.testing.assert_allclose(o[:, a, :], mean, atol=1e-12)


def test_gqa_equals_mha_with_repeated_kv_heads():
    rng = np.random.default_rng(4)
    q = rng.standard_normal((6, 6, 8))
    k = rng.standard_normal((6, 2, 8))
    v = rng.standard_normal((6, 2, 8))
    rep_k = np.repeat(k, 3, axis=1)     # head a -> kv head a // 3
    rep_v = np.repeat(v, 3, axis=1)
    np.testing.assert_allclose(decoder.causal_attention(q, k, v),
                               decoder.causal_attention(q, rep_k, rep_v), atol=1e-13)


def test_attention_q_pos_offsets():
    # a query at absolute position p against a longer key set sees keys 0..p
    rng = np.random.default_rng(5)
    q = rng.standard_normal((8, 2, 4))
    k = rng.standard_normal((8, 1, 4))
    v = rng.standard_normal((8, 1, 4))
    full = decoder.causal_attention(q, k, v)
    part = decoder.causal_attention(q[5:6], k, v, q_pos=[5])
    np.testing.assert_allclose(part[0], full[5], atol=1e-13)


# --------------------------------------------------------------------- rope
def test_rope_closed_form_two_dims():
    # d = 2: one pair, frequency theta**0 = 1: plain rotation by `pos` radians
    x = np.array([[[0.3, -1.1]], [[2.0, 0.5]]])
    y = decoder.rope(x, [0, 3], 1.0e4)
    np.testing.assert_allclose(y[0], x[0], atol=0)
    c, s = math.cos(3.0), math.sin(3.0)
    np.testing.assert_allclose(y[1, 0], [2.0 * c - 0.5 * s, 0.5 * c + 2.0 * s], atol=1e-14)


def test_rope_pairing_and_frequency():
    # d = 4: pairs (0,2) at frequency 1 and (1,3) at frequency theta**(-1/2)
    theta = 100.0
    x = np.array([[[1.0, 0.0, 0.0, 0.0]], [[0.0, 1.0, 0.0, 0.0]]])
    y = decoder.rope(x, [2, 2], theta)
    np.testing.assert_allclose(y[0, 0], [math.cos(2.0), 0, math.sin(2.0), 0], atol=1e-14)
    a = 2.0 * theta ** -0.5
    np.testing.assert_allclose(y[1, 0], [0, math.cos(a), 0, math.sin(a)], atol=1e-14)


def test_rope_preserves_norm_and_is_relative():
    rng = np.random.default_rng(6)
    q = rng.standard_normal((1, 3, 16))
    k = rng.standard_normal((1, 3, 16))
    for m, n in [(5, 2), (105, 102), (40, 37)]:
        qm = decoder.rope(q, [m], 1e4)
        kn = decoder.rope(k, [n], 1e4)
        np.testing.assert_allclose(np.linalg.norm(qm, axis=-1), np.linalg.norm(q, axis=-1),
                                   rtol=1e-13)
        dots = np.sum(qm * kn, axis=-1)
        if m == 5:
            ref = dots
        np.testing.assert_allclose(dots, ref, atol=1e-11)


# ------------------------------------------------------------------ rmsnorm
def test_rmsnorm_worked_example():
    y = decoder.rmsnorm(np.array([3.0, 4.0]), np.array([1.0, 2.0]), 0.0)
    r = math.sqrt(12.5)
    np.testing.assert_allclose(y, [3.0 / r, 8.0 / r], atol=1e-15)


def test_rmsnorm_unit_mean_square_and_scale_invariance():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((5, 64))
    g = np.ones(64)
    y = decoder.rmsnorm(x, g, 1e-12)
    np.testing.assert_allclose(np.mean(y * y, -1), 1.0, atol=1e-9)
    np.testing.assert_allclose(decoder.rmsnorm(7.5 * x, g, 1e-12), y, atol=1e-9)
    # eps sits inside the square root, added to the mean square
    y2 = decoder.rmsnorm(np.array([1.0, 1.0]), np.ones(2), 3.0)
    np.testing.assert_allclose(y2, [0.5, 0.5], atol=1e-15)


# ------------------------------------------------------------------- swiglu
def test_swiglu_matches_scalar_loops():
    rng = np.random.default_rng(8)
    H, F, T = 5, 7, 3
    u = rng.standard_normal((T, H))
    wg, wu, wd = rng.standard_normal((F, H)), rng.standard_normal((F, H)), rng.standard_normal((H, F))
    ref = np.zeros((T, H))
    for t in range(T):
        act = []
        for f in range(F):
            g = sum(u[t, i] * wg[f, i] for i in range(H))
            up = sum(u[t, i] * wu[f, i] for i in range(H))
            act.append(g / (1.0 + math.exp(-g)) * up)
        for o in range(H):
            ref[t, o] = sum(act[f] * wd[o, f] for f in range(F))
    np.testing.assert_allclose(decoder.swiglu_ffn(u, wg, wu, wd), ref, atol=1e-12)


# -------------------------------------------------------------- whole model
@pytest.fixture(scope="module")
def tiny():
    cfg = synth.shape("tiny")
    w = synth.random_gains(synth.make_weights(cfg, 0, qkv_bias=True, std=0.05), 11)
    return cfg, w


def test_forward_rows_equal_plain_definition(tiny):
    cfg, w = tiny
    toks = np.random.default_rng(9).integers(0, cfg["vocab"], 12)
    allrows = decoder.forward(toks, w, cfg)
    for t in (0, 5, 11):
        np.testing.assert_allclose(allrows[t], decoder.next_logits(toks[: t + 1], w, cfg),
                                   atol=1e-11)


def test_incremental_kv_equals_full_recompute(tiny):
    cfg, w = tiny
    toks = np.random.default_rng(10).integers(0, cfg["vocab"], 20)
    dec = decoder.IncrementalDecoder(w, cfg)
    got = [dec.append(toks[:7])]
    for t in range(7, 20):
        got.append(dec.append(toks[t]))
    want = decoder.forward(toks, w, cfg)[6:]
    np.testing.assert_allclose(np.stack(got), want, atol=1e-11)


def test_forward_matches_public_qwen2_implementation():
    """The whole composition (pre-norm blocks, rotate-half RoPE, GQA mapping,
    eps placement, SwiGLU, QKV bias, untied head) against the Qwen2 model class
    of the `transformers` library in float64 on random weights."""
    torch = pytest.importorskip("torch")
    tf = pytest.importorskip("transformers")
    cfg = synth.shape("tiny", n_layers=2, hidden=48, n_q_heads=6, n_kv_heads=2, head_dim=8,
                      ffn=56, vocab=96, rope_theta=1.0e4, rms_eps=1.0e-6)
    w = synth.random_gains(synth.make_weights(cfg, 3, qkv_bias=True, std=0.3), 5)
    hc = tf.Qwen2Config(vocab_size=cfg["vocab"], hidden_size=cfg["hidden"],
                        intermediate_size=cfg["ffn"], num_hidden_layers=cfg["n_layers"],
                        num_attention_heads=cfg["n_q_heads"],
                        num_key_value_heads=cfg["n_kv_heads"], max_position_embeddings=256,
                        rope_theta=cfg["rope_theta"], rms_norm_eps=cfg["rms_eps"],
                        tie_word_embeddings=False, attn_implementation="eager",
                        use_sliding_window=False)
    model = tf.Qwen2ForCausalLM(hc).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "model.norm.weight": w["final_norm"],
          "lm_head.weight": w["lm_head"]}
    names = dict(wq="self_attn.q_proj.weight", wk="self_attn.k_proj.weight",
                 wv="self_attn.v_proj.weight", wo="self_attn.o_proj.weight",
                 bq="self_attn.q_proj.bias", bk="self_attn.k_proj.bias",
                 bv="self_attn.v_proj.bias", wgate="mlp.gate_proj.weight",
                 wup="mlp.up_proj.weight", wdown="mlp.down_proj.weight",
                 norm_attn="input_layernorm.weight", norm_ffn="post_attention_layernorm.weight")
    for l, lw in enumerate(w["layers"]):
        for k, n in names.items():
            sd[f"model.layers.{l}.{n}"] = lw[k]
    sd = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in sd.items()}
    missing, unexpected = model.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in m or "inv_freq" in m for m in missing), (missing, unexpected)
    toks = np.random.default_rng(12).integers(0, cfg["vocab"], 37)
    with torch.no_grad():
        ref = model(torch.from_numpy(toks)[None]).logits[0].numpy()
    got = decoder.forward(toks, w, cfg)
    assert np.abs(ref).max() > 0.5          # the comparison is not vacuous
    # the library evaluates the rotary angles in float32 even in a float64
    # model, which alone moves logits by ~5e-6; any structural mistake (pairing,
    # head mapping, eps, bias, gain) moves them by more than 1e-2
    np.testing.assert_allclose(got, ref, atol=3e-5)
