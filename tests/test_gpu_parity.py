"""GPU parity: the HIP library (through the C ABI) against the CPU oracle on
identical seeded inputs.  Tolerances are the ones the build is held to:
logits max-abs error <= 2e-2, per-token log-prob error <= 1e-2 (half-precision
matrix operands and K/V, float32 accumulation); sampled token ids bit-exact given identical
float32 logits and seed."""
import numpy as np
import pytest

from paper_2505_24298_amd import synth

pytestmark = pytest.mark.gpu

LOGIT_TOL = 2e-2
LOGP_TOL = 1e-2


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


@pytest.fixture(scope="module")
def binding():
    from paper_2505_24298_amd import binding
    binding.lib()
    return binding


def _f16(a):
    return np.asarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)


def _f16_weights(w):
    """The values the GPU computes with: float32 parameters rounded to half
    precision (nearest even), as the library does when it receives them."""
    out = dict(embed=_f16(w["embed"]), lm_head=_f16(w["lm_head"]), final_norm=_f16(w["final_norm"]),
               layers=[])
    for lw in w["layers"]:
        out["layers"].append({k: _f16(v) for k, v in lw.items()})
    return out


def _teacher_forced_run(torch, binding, cfg, w_f32, prompts, n_new, *, qkv_bias=False, seed=0,
                        temperature=1.0, top_p=1.0, max_batch_tokens=64, interrupt=None,
                        kv_blocks=256, shuffle_ids=None):
    """Oracle free-runs; the GPU is fed the oracle's tokens.  Returns the worst
    logits and log-prob deviations.  `interrupt` = (step, new fp32 weights)."""
    from oracle import rollout
    ids = list(range(len(prompts))) if shuffle_ids is None else list(shuffle_ids)
    wk = rollout.RolloutWorker(cfg, _f16_weights(w_f32), version=0, seed=seed,
                               temperature=temperature, top_p=top_p)
    for s, p in zip(ids, prompts):
        wk.add(s, p)
    eng = binding.Areal(cfg, max_seqs=max(ids) + 1, max_seq_len=max(len(p) for p in prompts) + n_new + 1,
                        max_batch_tokens=max_batch_tokens, kv_blocks=kv_blocks, convert_weights=True)
    eng.load_weights(binding.weights_to_device(w_f32, bf16=False), 0)
    logits = eng.prefill(ids, prompts)
    worst_logit, worst_lb, worst_lf = 0.0, 0.0, 0.0
    version = 0
    for step in range(n_new):
        if interrupt is not None and step == interrupt[0]:
            version += 1
            wk.update_weights(_f16_weights(interrupt[1]), version)
            live, logits, retok = eng.update_weights_interrupt(
                binding.weights_to_device(interrupt[1], bf16=False), version)
            assert live.tolist() == sorted(ids)
            assert retok == sum(len(wk.tokens[s]) for s in ids)
            order = [sorted(ids).index(s) for s in ids]
            logits = logits[torch.tensor(order, device=logits.device)].contiguous()
        positions = [len(wk.tokens[s]) for s in ids]
        ref_logits, ref_tok = wk.step(ids)                       # oracle samples its own tokens
        got = logits.cpu().numpy()
        worst_logit = max(worst_logit, float(np.abs(got - ref_logits).max()))
        forced = torch.from_numpy(ref_tok).to(logits.device)
        toks, lb, lf = eng.sample_logprob(logits, ids, positions, temperature, top_p, seed,
                                          forced_tokens=forced)
        assert toks.cpu().numpy().tolist() == ref_tok.tolist()
        ref_lb = np.array([wk.logp_behav[s][-1] for s in ids])
        ref_lf = np.array([wk.logp_full[s][-1] for s in ids])
        worst_lb = max(worst_lb, float(np.abs(lb.cpu().numpy() - ref_lb).max()))
        worst_lf = max(worst_lf, float(np.abs(lf.cpu().numpy() - ref_lf).max()))
        # free draw on the GPU's own logits must equal the oracle sampler on the same logits
        from oracle import sampler
        dt, _, _ = eng.sample_logprob(logits, ids, positions, temperature, top_p, seed)
        want, _, _ = sampler.sample_batch(got, temperature, top_p, seed, ids, positions)
        assert dt.cpu().numpy().tolist() == want.tolist()
        logits = eng.decode_step(ids, toks)
    # state the library keeps on the host and device
    for s in ids:
        assert eng.get_tokens(s).tolist() == wk.tokens[s]
        v = eng.get_versions(s)
        assert v[: wk.prompt_len[s]].tolist() == [-1] * wk.prompt_len[s]
        assert v[wk.prompt_len[s]:].tolist() == wk.versions[s]
    eng.close()
    return worst_logit, worst_lb, worst_lf


def test_tiny_config_teacher_forced(torch, binding):
    """Config "tiny": 8 sequences, prompts of 8-32 tokens, 64 generated tokens."""
    cfg, wl, prompts, outs = synth.make_workload("tiny")
    w = synth.make_weights(cfg, 0)
    dl, dlb, dlf = _teacher_forced_run(torch, binding, cfg, w, prompts, int(outs[0]))
    print(f"tiny: logits {dl:.2e}  logp_behav {dlb:.2e}  logp_full {dlf:.2e}")
    assert dl <= LOGIT_TOL and dlb <= LOGP_TOL and dlf <= LOGP_TOL


def test_tiny_bias_gains_large_values_chunked_prefill(torch, binding):
    """QKV bias, non-unit gains, larger weights (logits of order 1), prompts
    longer than one pass (chunked prefill across sequence boundaries), ids not
    in order."""
    cfg = synth.shape("tiny")
    w = synth.random_gains(synth.make_weights(cfg, 3, qkv_bias=True, std=0.05), 4)
    prompts = synth.make_prompts(cfg, 5, 1, 40, 150, seed=5)
    dl, dlb, dlf = _teacher_forced_run(torch, binding, cfg, w, prompts, 20, max_batch_tokens=64,
                                       shuffle_ids=[6, 2, 9, 0, 4])
    print(f"tiny/bias: logits {dl:.2e}  logp_behav {dlb:.2e}  logp_full {dlf:.2e}")
    assert dl <= LOGIT_TOL and dlb <= LOGP_TOL and dlf <= LOGP_TOL


def test_tiny_interrupt_matches_fresh_prefill_under_new_weights(torch, binding):
    cfg = synth.shape("tiny")
    w = synth.make_weights(cfg, 0)
    w2 = synth.perturb_weights(w, 1000, scale=5e-3, round_bf16=False)
    prompts = synth.make_prompts(cfg, 4, 1, 8, 40, seed=6)
    dl, dlb, dlf = _teacher_forced_run(torch, binding, cfg, w, prompts, 40, interrupt=(17, w2),
                                       max_batch_tokens=48)
    print(f"tiny/interrupt: logits {dl:.2e}  logp_behav {dlb:.2e}  logp_full {dlf:.2e}")
    assert dl <= LOGIT_TOL and dlb <= LOGP_TOL and dlf <= LOGP_TOL


def test_tiny_long_context_split_kv_decode(torch, binding):
    """Contexts of several hundred tokens: decode attention is cut into KV splits
    that are combined inside the kernel; prefill runs in several passes."""
    cfg = synth.shape("tiny")
    w = synth.make_weights(cfg, 2)
    prompts = synth.make_prompts(cfg, 3, 1, 300, 700, seed=9)
    dl, dlb, dlf = _teacher_forced_run(torch, binding, cfg, w, prompts, 6, max_batch_tokens=256,
                                       kv_blocks=160)
    print(f"tiny/long: logits {dl:.2e}  logp_behav {dlb:.2e}  logp_full {dlf:.2e}")
    assert dl <= LOGIT_TOL and dlb <= LOGP_TOL and dlf <= LOGP_TOL


def test_top_p_temperature_teacher_forced(torch, binding):
    cfg = synth.shape("tiny")
    w = synth.make_weights(cfg, 8)
    prompts = synth.make_prompts(cfg, 3, 2, 8, 24, seed=7)
    dl, dlb, dlf = _teacher_forced_run(torch, binding, cfg, w, prompts, 24, temperature=0.6, top_p=0.95,
                                       seed=(5 << 32) | 77)
    print(f"tiny/top-p: logits {dl:.2e}  logp_behav {dlb:.2e}  logp_full {dlf:.2e}")
    assert dl <= LOGIT_TOL and dlb <= LOGP_TOL and dlf <= LOGP_TOL


def test_errors_leave_state_unchanged(torch, binding):
    cfg = synth.shape("tiny")
    eng = binding.Areal(cfg, max_seqs=4, max_seq_len=64, max_batch_tokens=32, kv_blocks=3,
                        convert_weights=True)
    p = [np.arange(20, dtype=np.int32)]
    with pytest.raises(binding.ArealError) as e:
        eng.prefill([0], p)
    assert e.value.code == binding.E_STATE                       # no weights yet
    eng.load_weights(binding.weights_to_device(synth.make_weights(cfg, 0), bf16=False), 0)
    eng.prefill([0], p)                                          # 2 of 3 blocks
    total, free = eng.kv_blocks()
    assert (total, free) == (3, 1)
    with pytest.raises(binding.ArealError) as e:
        eng.prefill([1], [p[0] + 1])                             # another prompt: needs 2 blocks, 1 free
    assert e.value.code == binding.E_NOMEM and eng.kv_blocks() == (3, 1) and eng.seq_len(1) == -1
    with pytest.raises(binding.ArealError) as e:
        eng.prefill([0], p)                                      # id already live
    assert e.value.code == binding.E_INVAL
    with pytest.raises(binding.ArealError) as e:
        eng.prefill([2], [np.array([5000], dtype=np.int32)])     # token outside the vocabulary
    assert e.value.code == binding.E_INVAL
    tok = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.ArealError) as e:
        eng.decode_step([3], tok)                                # never prefilled
    assert e.value.code == binding.E_STATE
    lg = torch.zeros((1, cfg["vocab"]), device="cuda")
    with pytest.raises(binding.ArealError) as e:
        eng.sample_logprob(lg, [0], [0], temperature=0.0)
    assert e.value.code == binding.E_INVAL
    eng.free_seq(0)
    assert eng.kv_blocks() == (3, 3)
    eng.close()


def test_tiny_deep_context_many_splits(torch, binding):
    """One sequence of 8,300 tokens on the tiny shape: 33 splits of 256 tokens
    would exceed the split limit, so the launch takes longer splits; prefill runs
    in many passes over one long sequence."""
    from oracle import decoder
    cfg = synth.shape("tiny")
    w = synth.make_weights(cfg, 17)
    rng = np.random.default_rng(18)
    T = 8300
    prompt = rng.integers(0, cfg["vocab"], size=T).astype(np.int32)
    nxt = rng.integers(0, cfg["vocab"], size=3).astype(np.int32)
    eng = binding.Areal(cfg, max_seqs=1, max_seq_len=T + 8, max_batch_tokens=1024, kv_blocks=T // 16 + 4,
                        convert_weights=True)
    eng.load_weights(binding.weights_to_device(w, bf16=False), 0)
    got = [eng.prefill([0], [prompt]).cpu().numpy()[0]]
    for t in range(3):
        got.append(eng.decode_step([0], torch.from_numpy(nxt[t:t + 1].copy()).cuda()).cpu().numpy()[0])
    eng.close()
    seq = np.concatenate([prompt, nxt])
    ref = decoder.forward(seq, _f16_weights(w), cfg, rows=[T - 1, T, T + 1, T + 2])
    worst = max(float(np.abs(g - r).max()) for g, r in zip(got, ref))
    print(f"tiny/deep: logits {worst:.2e}")
    assert worst <= LOGIT_TOL


@pytest.mark.parametrize("nq,nkv,d", [(4, 2, 64), (2, 2, 32), (16, 1, 32), (14, 2, 64), (8, 1, 128)])
def test_head_geometries(torch, binding, nq, nkv, d):
    """Head dimensions 32 / 64 / 128 and query-per-KV-head groups of 1, 2, 7, 8
    and 16 (every attention template and row-group count): prompts long enough
    for several prefill tiles and KV splits, an interrupt in the middle."""
    cfg = synth.shape("tiny", n_q_heads=nq, n_kv_heads=nkv, head_dim=d, hidden=128, ffn=192)
    w = synth.random_gains(synth.make_weights(cfg, 40 + nq, qkv_bias=True, std=0.04), 7)
    w2 = synth.perturb_weights(w, 1003, scale=5e-3, round_bf16=False)
    prompts = synth.make_prompts(cfg, 3, 1, 30, 330, seed=nq + d)
    dl, dlb, dlf = _teacher_forced_run(torch, binding, cfg, w, prompts, 12, qkv_bias=True, interrupt=(5, w2),
                                       max_batch_tokens=96, kv_blocks=96)
    print(f"heads {nq}/{nkv} d{d}: logits {dl:.2e}  logp_behav {dlb:.2e}  logp_full {dlf:.2e}")
    assert dl <= LOGIT_TOL and dlb <= LOGP_TOL and dlf <= LOGP_TOL


@pytest.mark.parametrize("hidden,ffn", [(200, 344), (4608, 320), (8192, 192)])
def test_hidden_sizes(torch, binding, hidden, ffn):
    """Hidden sizes off the 64-wide K slabs (register-staged GEMM path for every
    product) and in the two widest RMSNorm variants (rows of 4608 and 8192)."""
    cfg = synth.shape("tiny", hidden=hidden, ffn=ffn, n_layers=1)
    w = synth.random_gains(synth.make_weights(cfg, 50, std=0.02), 8)
    prompts = synth.make_prompts(cfg, 2, 1, 20, 70, seed=hidden)
    dl, dlb, dlf = _teacher_forced_run(torch, binding, cfg, w, prompts, 6, max_batch_tokens=64, kv_blocks=16)
    print(f"hidden {hidden}: logits {dl:.2e}  logp_behav {dlb:.2e}  logp_full {dlf:.2e}")
    assert dl <= LOGIT_TOL and dlb <= LOGP_TOL and dlf <= LOGP_TOL
