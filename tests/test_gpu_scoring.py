"""GPU parity of the teacher-forced log-prob pass (proximal-policy term of
Eq. 5) against oracle/scoring.py, through the C ABI; and its agreement with the
behaviour log-probs the GPU rollout emitted for the same trajectories."""
import numpy as np
import pytest

from paper_2505_24298_amd import synth

pytestmark = pytest.mark.gpu

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
    out = dict(embed=_f16(w["embed"]), lm_head=_f16(w["lm_head"]), final_norm=_f16(w["final_norm"]),
               layers=[])
    for lw in w["layers"]:
        out["layers"].append({k: _f16(v) for k, v in lw.items()})
    return out


def _engine(binding, cfg, w, **kw):
    args = dict(max_seqs=4, max_seq_len=320, max_batch_tokens=64, kv_blocks=64, convert_weights=True)
    args.update(kw)
    eng = binding.Areal(cfg, **args)
    eng.load_weights(binding.weights_to_device(w, bf16=False), 0)
    return eng


@pytest.mark.parametrize("temperature,scratch_rows", [(1.0, 16), (0.6, 1), (1.3, 500)])
def test_packed_sequences_match_oracle(torch, binding, temperature, scratch_rows):
    """Lengths 1, 2, one block, across blocks, longer than one pass; more
    sequences than free slots (several groups); scratch smaller / larger than a pass."""
    from oracle import scoring
    cfg = synth.shape("tiny")
    w = synth.random_gains(synth.make_weights(cfg, 21, qkv_bias=True, std=0.05), 3)
    rng = np.random.default_rng(8)
    lens = [1, 2, 16, 17, 45, 150, 64, 3, 300]
    seqs = [rng.integers(0, cfg["vocab"], size=n).astype(np.int32) for n in lens]
    eng = _engine(binding, cfg, w)
    got = eng.recompute_logprob(seqs, temperature, scratch_rows).cpu().numpy()
    ref = scoring.batch_logprobs(seqs, _f16_weights(w), cfg, temperature)
    assert got.shape == ref.shape
    cu = np.concatenate([[0], np.cumsum(lens)])
    assert np.all(got[cu[:-1]] == 0.0)
    err = np.abs(got - ref).max()
    print(f"scoring T={temperature}: max |dlogp| {err:.2e}")
    assert err <= LOGP_TOL
    assert eng.kv_blocks() == (64, 64)                     # borrowed blocks returned
    eng.close()


@pytest.mark.parametrize("vocab,scratch_rows", [(1024, 64), (1000, 700), (5000, 3)])
def test_large_passes_fused_and_unfused_output_projection(torch, binding, vocab, scratch_rows):
    """Passes of up to 1,000 rows: the output projection folds the log-sum-exp into its epilogue
    (256 x 256 tiles above 256 rows, 128 x 128 below, as many rows per launch as their per-tile
    pairs fit into the scratch), with vocabularies that end inside a tile.  Against the oracle,
    and against the path that writes the logits of a chunk of rows and reduces them afterwards."""
    import os
    from oracle import scoring
    cfg = synth.shape("tiny", vocab=vocab)
    w = synth.random_gains(synth.make_weights(cfg, 23, qkv_bias=True, std=0.05), 3)
    rng = np.random.default_rng(vocab)
    lens = [700, 290, 5, 257, 130, 1, 64]
    seqs = [rng.integers(0, vocab, size=n).astype(np.int32) for n in lens]
    ref = scoring.batch_logprobs(seqs, _f16_weights(w), cfg, 0.8)
    got = {}
    saved = os.environ.get("AREAL_SCORE_FUSED")
    try:
        for fused in ("1", "0"):
            os.environ["AREAL_SCORE_FUSED"] = fused
            eng = _engine(binding, cfg, w, max_seqs=4, max_seq_len=704, max_batch_tokens=1000, kv_blocks=200)
            got[fused] = eng.recompute_logprob(seqs, 0.8, scratch_rows).cpu().numpy()
            assert eng.kv_blocks() == (200, 200)
            eng.close()
            err = np.abs(got[fused] - ref).max()
            print(f"vocab {vocab}, fused {fused}: max |dlogp| {err:.2e}")
            assert err <= LOGP_TOL
    finally:
        if saved is None:
            os.environ.pop("AREAL_SCORE_FUSED", None)
        else:
            os.environ["AREAL_SCORE_FUSED"] = saved
    assert np.abs(got["1"] - got["0"]).max() <= 2e-3        # two runs differ by the order of float32 atomic adds


def test_scoring_leaves_live_sequences_alone_and_matches_emitted_logprobs(torch, binding):
    """Generate on the GPU, then score the finished trajectories while other
    sequences are still live: (a) the recomputed log-probs equal the untruncated
    log-probs emitted at sampling time (same weights), (b) the live sequences go
    on exactly as the oracle says."""
    from oracle import rollout
    cfg = synth.shape("tiny")
    w = synth.make_weights(cfg, 22, std=0.05)
    prompts = synth.make_prompts(cfg, 3, 1, 6, 30, seed=2)
    ids = [0, 1, 2]
    eng = _engine(binding, cfg, w, kv_blocks=40)
    wk = rollout.RolloutWorker(cfg, _f16_weights(w), version=0, seed=3)
    for s, p in zip(ids, prompts):
        wk.add(s, p)
    logits = eng.prefill(ids, prompts)
    emitted = {s: [] for s in ids}
    for step in range(25):
        positions = [len(wk.tokens[s]) for s in ids]
        ref_logits, ref_tok = wk.step(ids)
        forced = torch.from_numpy(ref_tok).to(logits.device)
        toks, lb, lf = eng.sample_logprob(logits, ids, positions, 1.0, 1.0, 3, forced_tokens=forced)
        for i, s in enumerate(ids):
            emitted[s].append(float(lf[i]))
        logits = eng.decode_step(ids, toks)
    # sequences 0 and 1 "finish": score them (sequence 2 stays live, one slot is free)
    done = [eng.get_tokens(0), eng.get_tokens(1)]
    eng.free_seq(0)
    used_before = eng.kv_blocks()
    lp = eng.recompute_logprob(done, 1.0, 32).cpu().numpy()
    assert eng.kv_blocks() == used_before
    off = 0
    for s, toks_s in zip((0, 1), done):
        n_p = wk.prompt_len[s]
        got = lp[off + n_p: off + len(toks_s)]
        assert np.abs(got - np.array(emitted[s])).max() <= 5e-3
        off += len(toks_s)
    # the live sequence continues unharmed
    positions = [len(wk.tokens[2])]
    ref_logits, ref_tok = wk.step([2])
    assert np.abs(logits[2:3].cpu().numpy() - ref_logits).max() <= 2e-2
    nxt = eng.decode_step([2], torch.from_numpy(ref_tok).to(logits.device))
    ref_logits2, _ = wk.step([2])
    assert np.abs(nxt.cpu().numpy() - ref_logits2).max() <= 2e-2
    eng.close()


def test_scoring_errors(torch, binding):
    cfg = synth.shape("tiny")
    w = synth.make_weights(cfg, 23)
    eng = _engine(binding, cfg, w, max_seqs=1, max_seq_len=64, kv_blocks=2)
    seq = np.arange(20, dtype=np.int32)
    assert eng.recompute_logprob([], 1.0).numel() == 0
    with pytest.raises(binding.ArealError) as e:
        eng.recompute_logprob([seq], 0.0)
    assert e.value.code == binding.E_INVAL
    with pytest.raises(binding.ArealError) as e:
        eng.recompute_logprob([np.arange(40, dtype=np.int32)], 1.0)      # 3 blocks, 2 in the pool
    assert e.value.code == binding.E_NOMEM
    eng.prefill([0], [seq])
    with pytest.raises(binding.ArealError) as e:
        eng.recompute_logprob([seq], 1.0)                                # the only slot is live
    assert e.value.code == binding.E_NOMEM
    assert eng.seq_len(0) == 20 and eng.kv_blocks() == (2, 0)
    eng.close()


def test_ppo_objective_matches_oracle(torch, binding):
    """Decoupled PPO objective (Eq. 5) over 100,003 tokens (several work-groups,
    a ragged tail), with and without a mask, against the float64 oracle."""
    from oracle import trainer_side
    cfg = synth.shape("tiny")
    eng = _engine(binding, cfg, synth.make_weights(cfg, 0))
    rng = np.random.default_rng(5)
    n = 100003
    lt, lp, lb = (rng.normal(-3.0, 0.7, n).astype(np.float32) for _ in range(3))
    adv = rng.normal(0.0, 1.0, n).astype(np.float32)
    mask = (rng.random(n) < 0.8).astype(np.uint8)
    dev = lambda a: torch.from_numpy(a).cuda()
    for m in (None, mask):
        (total, n_clip, n_cnt), obj = eng.ppo_objective(dev(lt), dev(lp), dev(lb), dev(adv), 0.2,
                                                        mask=None if m is None else dev(m), per_token=True)
        want_total, want_obj, want_clip = trainer_side.decoupled_ppo_objective(lt, lp, lb, adv, 0.2, mask=m)
        assert np.abs(obj.cpu().numpy() - want_obj).max() <= 1e-4 * max(1.0, np.abs(want_obj).max())
        assert abs(total - want_total) <= 1e-5 * np.abs(want_obj).sum()
        assert n_cnt == (n if m is None else int(m.sum()))
        assert abs(n_clip - int(want_clip.sum())) <= 3          # ties at the clip edge may round either way
    (total, n_clip, n_cnt), _ = eng.ppo_objective(dev(lt[:0]), dev(lp[:0]), dev(lb[:0]), dev(adv[:0]), 0.2)
    assert (total, n_clip, n_cnt) == (0.0, 0, 0)
    eng.close()
