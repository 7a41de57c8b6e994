"""Pins for oracle/scoring.py (token log-probabilities of whole trajectories,
the proximal-policy term of Eq. 5): normalisation by enumeration, the direction
of the one-token shift on a model built to copy a permutation, a closed form,
the cross-entropy loss of the public Qwen2 implementation, and agreement with
the log-probs the rollout oracle emits while generating."""
import math

import numpy as np
import pytest

from oracle import rollout, scoring
from paper_2505_24298_amd import synth


def _tiny(**kw):
    base = dict(n_layers=2, hidden=32, n_q_heads=4, n_kv_heads=2, head_dim=8, ffn=40, vocab=24,
                rope_theta=1.0e4, rms_eps=1.0e-6)
    base.update(kw)
    return synth.shape("tiny", **base)


def test_probabilities_of_all_continuations_sum_to_one():
    """Replace the token at position t by every vocabulary entry in turn: the
    probabilities the oracle reports for position t must add up to 1."""
    cfg = _tiny()
    w = synth.make_weights(cfg, 1, std=0.4)
    toks = np.random.default_rng(0).integers(0, cfg["vocab"], 9)
    for t in (1, 4, 8):
        for T in (1.0, 0.6):
            total = 0.0
            for cand in range(cfg["vocab"]):
                x = toks.copy()
                x[t] = cand
                total += math.exp(scoring.sequence_logprobs(x[: t + 1], w, cfg, T)[t])
            assert abs(total - 1.0) < 1e-12


def test_shift_direction_on_a_permutation_copier():
    """Zero layers, one-hot embeddings, an output projection that sends token a
    to (a+1) mod V with a large margin: a sequence that follows the cycle has
    log-prob ~ 0 at every position, one that runs backwards is far below."""
    V = 8
    cfg = _tiny(n_layers=0, hidden=V, vocab=V)
    w = synth.make_weights(cfg, 0)
    w["embed"] = np.eye(V)
    w["final_norm"] = np.ones(V)
    lm = np.zeros((V, V))
    for a in range(V):
        lm[(a + 1) % V, a] = 20.0          # logits = rmsnorm(e_a) . lm^T; rmsnorm(e_a) = sqrt(V) e_a
    w["lm_head"] = lm
    w["layers"] = []
    fwd = np.arange(0, 6) % V
    lp = scoring.sequence_logprobs(fwd, w, cfg)
    assert lp[0] == 0.0 and np.all(lp[1:] > -1e-6)
    bwd = fwd[::-1].copy()
    assert np.all(scoring.sequence_logprobs(bwd, w, cfg)[1:] < -20.0)


def test_zero_output_projection_gives_uniform():
    cfg = _tiny()
    w = synth.make_weights(cfg, 2)
    w["lm_head"] = np.zeros_like(w["lm_head"])
    lp = scoring.sequence_logprobs([3, 1, 4, 1, 5], w, cfg, temperature=0.7)
    np.testing.assert_allclose(lp[1:], -math.log(cfg["vocab"]), atol=1e-14)
    assert lp[0] == 0.0
    assert scoring.sequence_logprobs([7], w, cfg).tolist() == [0.0]
    assert scoring.batch_logprobs([], w, cfg).shape == (0,)


def test_mean_negative_logprob_is_the_public_cross_entropy_loss():
    torch = pytest.importorskip("torch")
    tf = pytest.importorskip("transformers")
    cfg = _tiny(hidden=48, n_q_heads=6, ffn=56, vocab=96)
    w = synth.random_gains(synth.make_weights(cfg, 3, qkv_bias=True, std=0.3), 5)
    hc = tf.Qwen2Config(vocab_size=cfg["vocab"], hidden_size=cfg["hidden"], intermediate_size=cfg["ffn"],
                        num_hidden_layers=cfg["n_layers"], num_attention_heads=cfg["n_q_heads"],
                        num_key_value_heads=cfg["n_kv_heads"], max_position_embeddings=256,
                        rope_theta=cfg["rope_theta"], rms_norm_eps=cfg["rms_eps"], tie_word_embeddings=False,
                        attn_implementation="eager", use_sliding_window=False)
    model = tf.Qwen2ForCausalLM(hc).double().eval()
    sd = {"model.embed_tokens.weight": w["embed"], "model.norm.weight": w["final_norm"],
          "lm_head.weight": w["lm_head"]}
    names = dict(wq="self_attn.q_proj.weight", wk="self_attn.k_proj.weight", wv="self_attn.v_proj.weight",
                 wo="self_attn.o_proj.weight", bq="self_attn.q_proj.bias", bk="self_attn.k_proj.bias",
                 bv="self_attn.v_proj.bias", wgate="mlp.gate_proj.weight", wup="mlp.up_proj.weight",
                 wdown="mlp.down_proj.weight", norm_attn="input_layernorm.weight",
                 norm_ffn="post_attention_layernorm.weight")
    for l, lw in enumerate(w["layers"]):
        for k, n in names.items():
            sd[f"model.layers.{l}.{n}"] = lw[k]
    model.load_state_dict({k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in sd.items()},
                          strict=False)
    toks = np.random.default_rng(21).integers(0, cfg["vocab"], 29)
    with torch.no_grad():
        ids = torch.from_numpy(toks)[None]
        loss = float(model(ids, labels=ids).loss)          # mean over the 28 predicted tokens
    lp = scoring.sequence_logprobs(toks, w, cfg)
    assert loss > 1.0
    assert abs(-lp[1:].mean() - loss) < 3e-5               # rotary angles are float32 in the library


def test_recomputation_equals_the_log_probs_emitted_while_generating():
    """Unchanged weights: the log-prob of each generated token, recomputed over
    the finished trajectory, is the untruncated log-prob the rollout reported
    when it sampled that token (the sampler works on float32 logits)."""
    cfg = _tiny(vocab=64)
    w = synth.make_weights(cfg, 4, std=0.3)
    for T, top_p in ((1.0, 1.0), (0.6, 0.9)):
        wk = rollout.RolloutWorker(cfg, w, version=0, seed=5, temperature=T, top_p=top_p)
        prompt = [5, 9, 2, 40]
        wk.add(0, prompt)
        for _ in range(12):
            wk.step([0])
        lp = scoring.sequence_logprobs(wk.tokens[0], w, cfg, T)
        np.testing.assert_allclose(lp[len(prompt):], wk.logp_full[0], atol=2e-6)
