"""The streaming regime of bench.py (slots refilled as sequences finish, the
staleness gate, weight update + interrupt per finished training batch) on the
tiny shape: every trajectory is generated to its full length, the number of
weight updates is the number of training batches, the synchronous schedule
(eta = 0) never overlaps batches, a larger eta needs fewer decode steps, and for
every eta the run takes exactly the ticks of the oracle's plain event loop, with
every request submitted and completed under the versions that loop gives it."""
import numpy as np
import pytest

from oracle import staleness
from paper_2505_24298_amd import synth

pytestmark = pytest.mark.gpu


def _run(eta, n_total=48, slots=8, train_batch=8):
    import torch
    from paper_2505_24298_amd.harness import streaming_rollout
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
    # Section 5.1: the same stream through the oracle's controller, one request at a time
    ticks, done = staleness.simulate_stream(n_total, train_batch, eta, slots, outs)
    assert r["ticks"] == ticks
    assert sorted(r["records"]) == sorted(done)
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


@pytest.mark.parametrize("eta", [1, 2, 5])
def test_streaming_matches_the_oracle_event_loop(eta):
    _run(eta=eta)
