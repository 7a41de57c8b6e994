"""Pins for oracle/rollout.py: the generate / update_weights semantics."""
import numpy as np
import pytest

from oracle import decoder, rollout
from paper_2505_24298_amd import synth


@pytest.fixture(scope="module")
def setup():
    cfg, wl, prompts, outs = synth.make_workload("tiny")
    w = synth.make_weights(cfg, 0)
    return cfg, w, prompts


def _run(cfg, w, prompts, n_new, use_cache, interrupt_at=(), new_w=None, ids=None):
    ids = list(range(len(prompts))) if ids is None else ids
    wk = rollout.RolloutWorker(cfg, w, version=0, seed=0, use_cache=use_cache)
    for s, p in zip(ids, prompts):
        wk.add(s, p)
    logits = []
    for step in range(n_new):
        if step in interrupt_at:
            wk.update_weights(new_w if new_w is not None else wk.w, wk.version + 1)
        lg, _ = wk.step(ids)
        logits.append(lg)
    return wk, np.stack(logits)


def test_cached_worker_equals_plain_definition(setup):
    cfg, w, prompts = setup
    a, la = _run(cfg, w, prompts[:3], 12, use_cache=False)
    b, lb = _run(cfg, w, prompts[:3], 12, use_cache=True)
    assert a.tokens == b.tokens
    assert np.abs(la.astype(np.float64) - lb).max() <= 1e-5


def test_interrupt_with_unchanged_weights_is_invisible(setup):
    cfg, w, prompts = setup
    a, la = _run(cfg, w, prompts[:4], 16, use_cache=True)
    b, lb = _run(cfg, w, prompts[:4], 16, use_cache=True, interrupt_at=(5, 6, 11))
    assert a.tokens == b.tokens
    assert np.abs(la - lb).max() <= 1e-5
    assert a.logp_behav == b.logp_behav
    # version tags: monotone, change exactly at the interrupts
    for s in range(4):
        assert b.versions[s] == [0] * 5 + [1] * 1 + [2] * 5 + [3] * 5


def test_interrupt_with_new_weights_equals_fresh_prefill(setup):
    cfg, w, prompts = setup
    w2 = synth.perturb_weights(w, 1000, scale=5e-3, round_bf16=False)
    wk, _ = _run(cfg, w, prompts[:3], 6, use_cache=True)
    before = {s: (list(wk.tokens[s]), list(wk.logp_behav[s]), list(wk.versions[s])) for s in range(3)}
    wk.update_weights(w2, 1)
    for s in range(3):
        fresh = decoder.next_logits(wk.tokens[s], w2, cfg)
        old = decoder.next_logits(wk.tokens[s], w, cfg)
        np.testing.assert_allclose(wk.next_logits(s), fresh, atol=1e-10)
        assert np.abs(fresh - old).max() > 1e-4              # the weights did change
        assert (wk.tokens[s], wk.logp_behav[s], wk.versions[s]) == before[s]
    wk.step([0, 1, 2])
    assert all(wk.versions[s][-1] == 1 and wk.versions[s][:-1] == [0] * 6 for s in range(3))


def test_sequences_do_not_depend_on_batch_mates_or_order(setup):
    cfg, w, prompts = setup
    a, _ = _run(cfg, w, prompts[:4], 8, use_cache=False)
    b, _ = _run(cfg, w, [prompts[2]], 8, use_cache=False, ids=[2])
    assert a.tokens[2] == b.tokens[2] and a.logp_behav[2] == b.logp_behav[2]


def test_copies_of_a_prompt_diverge_by_seq_id(setup):
    cfg, w, prompts = setup
    a, _ = _run(cfg, w, [prompts[0], prompts[0]], 8, use_cache=False, ids=[0, 1])
    assert a.tokens[0][: len(prompts[0])] == a.tokens[1][: len(prompts[0])]
    assert a.tokens[0] != a.tokens[1]


def test_teacher_forcing_records_forced_tokens(setup):
    cfg, w, prompts = setup
    free, _ = _run(cfg, w, prompts[:2], 5, use_cache=False)
    wk = rollout.RolloutWorker(cfg, w, 0, seed=0)
    for s in range(2):
        wk.add(s, prompts[s])
    for t in range(5):
        forced = [free.tokens[s][len(prompts[s]) + t] for s in range(2)]
        wk.step([0, 1], forced=forced)
    assert wk.tokens == free.tokens and wk.logp_behav == free.logp_behav
