"""The streaming regime of bench.py (slots refilled as sequences finish, the
staleness gate, weight update + interrupt per finished training batch) on the
tiny shape: every trajectory is generated to its full length, the number of
weight updates is the number of training batches, the synchronous schedule
(eta = 0) never overlaps batches, and a larger eta needs fewer decode steps."""
import numpy as np
import pytest

from paper_2505_24298_amd import synth

pytestmark = pytest.mark.gpu


def _run(eta, n_total=48, slots=8, train_batch=8):
    import torch
    from bench import streaming_rollout
    from paper_2505_24298_amd import binding
    cfg = synth.shape("tiny")
    w0 = synth.make_weights(cfg, 0)
    w1 = synth.perturb_weights(w0, 1001, scale=1e-3, round_bf16=False)
    prompts = synth.make_prompts(cfg, n_total, 1, 4, 40, seed=3)
    outs = synth.output_lengths(n_total, 12, 1.0, 60, seed=4)
    eng = binding.Areal(cfg, max_seqs=slots, max_seq_len=128, max_batch_tokens=64, kv_blocks=slots * 9,
                        convert_weights=True)
    sets = [binding.weights_to_device(w0, bf16=False), binding.weights_to_device(w1, bf16=False)]
    eng.load_weights(sets[0], 0)
    r = streaming_rollout(eng, torch, cfg, binding.lib(), prompts, outs, slots, train_batch, eta, sets,
                          1.0, 1.0, 0)
    assert eng.kv_blocks()[0] == eng.kv_blocks()[1]            # every block returned
    eng.close()
    assert r["gen_tokens"] == int(outs.sum())
    assert r["interrupts"] == n_total // train_batch
    return r, outs


def test_streaming_completes_every_trajectory():
    sync, outs = _run(eta=0)
    # synchronous: batches never overlap, each takes as many steps as its longest output (minus the
    # last token of each sequence, which is sampled but not appended)
    per_batch = outs.reshape(-1, 8).max(axis=1) - 1
    assert sync["decode_steps"] == int(per_batch.sum())
    asyn, _ = _run(eta=3)
    assert asyn["decode_steps"] < sync["decode_steps"]
    assert asyn["mean_rows"] > sync["mean_rows"]
