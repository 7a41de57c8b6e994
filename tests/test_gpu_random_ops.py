"""Randomised differential test of the whole C ABI against the oracle: a seeded
sequence of admissions (with repeated prompts, so blocks get shared), ragged
decode steps, terminations, weight updates with re-prefill and scoring passes,
on the tiny shape.  After every operation that yields logits they are compared
with the oracle's plain recomputation; histories, version tags and the block
accounting are compared at the end of every round."""
import numpy as np
import pytest

from paper_2505_24298_amd import synth

pytestmark = pytest.mark.gpu

LOGIT_TOL = 2e-2


def _f16(a):
    return np.asarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)


def _f16_weights(w):
    out = dict(embed=_f16(w["embed"]), lm_head=_f16(w["lm_head"]), final_norm=_f16(w["final_norm"]), layers=[])
    for lw in w["layers"]:
        out["layers"].append({k: _f16(v) for k, v in lw.items()})
    return out


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_operation_sequences(seed):
    import torch
    from oracle import rollout, scoring
    from paper_2505_24298_amd import binding
    rng = np.random.default_rng(100 + seed)
    cfg = synth.shape("tiny")
    weights = [synth.make_weights(cfg, 70 + seed, qkv_bias=bool(seed & 1))]
    max_seqs, max_len, n_blocks = 6, 160, 48
    eng = binding.Areal(cfg, max_seqs=max_seqs, max_seq_len=max_len, max_batch_tokens=48, kv_blocks=n_blocks,
                        convert_weights=True)
    eng.load_weights(binding.weights_to_device(weights[0], bf16=False), 0)
    wk = rollout.RolloutWorker(cfg, _f16_weights(weights[0]), version=0, seed=seed)
    pool = [rng.integers(0, cfg["vocab"], size=int(n)).astype(np.int32) for n in (5, 16, 23, 40, 64)]
    live, pending = [], {}          # pending[s] = device logits row for the next token of s
    version = 0

    def check(ids, logits):
        ref = np.stack([wk.next_logits(s).astype(np.float32) for s in ids])
        assert np.abs(logits.cpu().numpy() - ref).max() <= LOGIT_TOL
        for i, s in enumerate(ids):
            pending[s] = logits[i:i + 1]

    for step in range(70):
        free_ids = [s for s in range(max_seqs) if s not in live]
        op = rng.choice(["admit", "decode", "decode", "decode", "free", "update", "score"])
        if op == "admit" and free_ids:
            k = int(rng.integers(1, len(free_ids) + 1))
            ids = [int(s) for s in rng.permutation(free_ids)[:k]]
            prompts = [pool[int(rng.integers(0, len(pool)))] for _ in ids]     # repeats share blocks
            need = sum((len(p) + 15) // 16 for p in prompts)
            if need > eng.kv_blocks()[1]:
                continue
            logits = eng.prefill(ids, prompts)
            for s, p in zip(ids, prompts):
                wk.finished.discard(s)
                wk.add(s, p)
                live.append(s)
            check(ids, logits)
        elif op == "decode" and live:
            k = int(rng.integers(1, len(live) + 1))
            ids = [int(s) for s in rng.permutation(live)[:k]]
            ids = [s for s in ids if len(wk.tokens[s]) + 1 < max_len]
            if not ids or eng.kv_blocks()[1] < len(ids):
                continue
            positions = [len(wk.tokens[s]) for s in ids]
            lg = torch.cat([pending[s] for s in ids])
            _, ref_tok = wk.step(ids)                      # the oracle draws from its own logits
            forced = torch.from_numpy(ref_tok).cuda()
            toks, _, _ = eng.sample_logprob(lg, ids, positions, 1.0, 1.0, seed, forced_tokens=forced)
            check(ids, eng.decode_step(ids, toks))
        elif op == "free" and live:
            s = int(rng.choice(live))
            eng.free_seq(s)
            wk.finish(s)
            live.remove(s)
            pending.pop(s, None)
        elif op == "update":
            version += 1
            w_new = synth.perturb_weights(weights[-1], 2000 + 10 * seed + version, scale=3e-3, round_bf16=False)
            weights.append(w_new)
            wk.update_weights(_f16_weights(w_new), version)
            got_live, logits, _ = eng.update_weights_interrupt(binding.weights_to_device(w_new, bf16=False), version)
            assert got_live.tolist() == sorted(live)
            if live:
                check(sorted(live), logits)
        elif op == "score" and len(live) < max_seqs:
            seqs = [np.asarray(wk.tokens[s], dtype=np.int32) for s in live[:2]] or [pool[2]]
            if sum((len(x) + 15) // 16 for x in seqs[:1]) > eng.kv_blocks()[1]:
                continue
            seqs = seqs[:1]
            before = eng.kv_blocks()
            got = eng.recompute_logprob(seqs, 1.0, scratch_rows=16).cpu().numpy()
            ref = scoring.batch_logprobs(seqs, wk.w, cfg, 1.0)
            assert np.abs(got - ref).max() <= 1e-2 and eng.kv_blocks() == before
        # state the library reports
        for s in live:
            assert eng.get_tokens(s).tolist() == wk.tokens[s]
            v = eng.get_versions(s)
            assert v[wk.prompt_len[s]:].tolist() == wk.versions[s]
    for s in list(live):
        eng.free_seq(s)
    assert eng.kv_blocks() == (n_blocks, n_blocks)
    eng.close()
