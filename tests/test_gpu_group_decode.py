"""Decode attention over prompt blocks that several live samples hold together
(Table 3: 16 answers per prompt): the leading blocks are walked once per set of
rows, every row keeps its own softmax state, and the merge folds the shared
partials into the row's own.  Logits against the oracle's plain full-sequence
forward (2e-2 as everywhere), with

* query groups of 6 and 7 at head_dim 128 (two sequences per MFMA tile), 2 at
  head_dim 32 (eight per tile) and 1 (sixteen per tile);
* a prompt of 300 tokens (five shared pieces of 64 tokens), one of 40 (two
  blocks), one of 17 (one block), one of 15 (no full block: nothing to share)
  and a prompt with a single sample;
* 16, 5, 2, 3 and 1 samples per prompt, so that sets hold full tiles, a
  half-filled tile and a single tile, and the 16 samples fill more than one set
  where a tile holds two sequences;
* samples that finish early, step by step, until a prompt has one live sample
  left (which then walks all its blocks itself);
* the same run with the sets switched off, which must agree with the first to
  rounding, and under the library's own rule (sets only while most of the
  context tokens a step reads are shared)."""
import os

import numpy as np
import pytest

from paper_2505_24298_amd import synth

pytestmark = pytest.mark.gpu

LOGIT_TOL = 2e-2
PROMPT_LENS = [300, 40, 17, 15, 33]
SAMPLES = [16, 5, 2, 3, 1]
N_DECODE = 6


def _f16(a):
    return np.asarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)


def _f16_weights(w):
    return dict(embed=_f16(w["embed"]), lm_head=_f16(w["lm_head"]), final_norm=_f16(w["final_norm"]),
                layers=[{k: _f16(v) for k, v in lw.items()} for lw in w["layers"]])


def _run(cfg, w, prompts_by_seq, forced, drop_at, groups_on):
    import torch
    from paper_2505_24298_amd import binding
    saved = {k: os.environ.get(k) for k in ("AREAL_DECODE_GROUPS", "AREAL_DECODE_MIN_CHUNK")}
    if groups_on is None:                  # the library's own rule: sets where most of the context read is shared
        os.environ.pop("AREAL_DECODE_GROUPS", None)
    else:
        os.environ["AREAL_DECODE_GROUPS"] = "1" if groups_on else "0"
    os.environ["AREAL_DECODE_MIN_CHUNK"] = "128"
    try:
        n = len(prompts_by_seq)
        eng = binding.Areal(cfg, max_seqs=n, max_seq_len=max(PROMPT_LENS) + N_DECODE + 8, max_batch_tokens=1024,
                            kv_blocks=n * 3 + sum(T // 16 + 1 for T in PROMPT_LENS) + 8, convert_weights=True)
        eng.load_weights(binding.weights_to_device(w, bf16=False), 0)
        ids = list(range(n))
        out = {0: dict(zip(ids, eng.prefill(ids, prompts_by_seq).cpu().numpy()))}
        live = list(ids)
        for t in range(N_DECODE):
            for i in drop_at.get(t, []):
                eng.free_seq(i)
                live.remove(i)
            toks = torch.from_numpy(np.array([forced[t, i] for i in live], dtype=np.int32)).cuda()
            out[t + 1] = dict(zip(live, eng.decode_step(live, toks).cpu().numpy()))
        counters = eng.decode_set_counters()
        eng.close()
        return out, counters
    finally:
        for k, v in saved.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v


@pytest.mark.parametrize("nq,nkv,d", [(6, 1, 128), (14, 2, 128), (4, 2, 32), (4, 4, 32)])
def test_shared_prompt_blocks_walked_once_per_set(nq, nkv, d):
    from oracle import decoder
    cfg = synth.shape("tiny", n_layers=2 if d == 32 else 1, n_q_heads=nq, n_kv_heads=nkv, head_dim=d,
                      hidden=256 if d == 128 else 64, ffn=512 if d == 128 else 128, rope_theta=1.0e6)
    w = synth.random_gains(synth.make_weights(cfg, 300 + nq, qkv_bias=True, std=0.03), 5)
    rng = np.random.default_rng(nq * 10 + nkv)
    prompts = [rng.integers(0, cfg["vocab"], size=T).astype(np.int32) for T in PROMPT_LENS]
    prompt_of = [p for p, k in enumerate(SAMPLES) for _ in range(k)]
    order = rng.permutation(len(prompt_of))                  # the samples of a prompt are not neighbours
    prompt_of = [prompt_of[j] for j in order]
    n = len(prompt_of)
    forced = rng.integers(0, cfg["vocab"], size=(N_DECODE, n)).astype(np.int32)
    # early terminations: the samples of prompt 0 leave two, three, ... at a time until one is left;
    # prompt 1 loses one per step
    of0 = [i for i in range(n) if prompt_of[i] == 0]
    of1 = [i for i in range(n) if prompt_of[i] == 1]
    drop_at = {1: of0[:2] + of1[:1], 2: of0[2:5] + of1[1:2], 3: of0[5:9] + of1[2:3], 4: of0[9:14] + of1[3:4],
               5: of0[14:15]}
    gone_after = {i: t for t, rows in drop_at.items() for i in rows}
    w16 = _f16_weights(w)
    ref = {}
    for i in range(n):
        steps = gone_after.get(i, N_DECODE)
        seq = np.concatenate([prompts[prompt_of[i]], forced[:steps, i]])
        T = PROMPT_LENS[prompt_of[i]]
        ref[i] = decoder.forward(seq, w16, cfg, rows=list(range(T - 1, T + steps)))
    by_seq = [prompts[p] for p in prompt_of]
    runs = {}
    for groups_on in (True, False, None):
        print(f"heads {nq}/{nkv} d={d} sets {groups_on}", flush=True)
        got, counters = _run(cfg, w, by_seq, forced, drop_at, groups_on)
        # what the sets must have covered: per step, every prompt with a full block and two live samples
        rows = row_tokens = set_tokens = 0
        for t in range(N_DECODE):
            for p, T in enumerate(PROMPT_LENS):
                live_p = sum(1 for i in range(n) if prompt_of[i] == p and gone_after.get(i, N_DECODE) > t)
                if groups_on and live_p >= 2 and T >= 16:
                    per_set = 4 * (16 // (nq // nkv))
                    rows += live_p
                    row_tokens += live_p * ((T - 1) // 16 * 16)
                    set_tokens += -(-live_p // per_set) * ((T - 1) // 16 * 16)
        if groups_on is None:
            # 84 % of the context tokens of the first steps are shared (the 16 samples of the 300-token
            # prompt), less once most of them have finished: some steps with sets, some without
            assert 0 < counters[0] < runs[True][1][0]
        else:
            assert counters == (rows, row_tokens, set_tokens)
        worst = 0.0
        for t, rows in got.items():
            for i, logits in rows.items():
                worst = max(worst, float(np.abs(logits - ref[i][t]).max()))
        print(f"  logits against the oracle {worst:.2e}", flush=True)
        assert worst <= LOGIT_TOL
        runs[groups_on] = (got, counters)
    diff = max(float(np.abs(runs[True][0][t][i] - runs[False][0][t][i]).max())
               for t in runs[True][0] for i in runs[True][0][t])
    print(f"  sets on against off {diff:.2e}", flush=True)
    assert diff <= 2e-3


@pytest.mark.parametrize("T", [2000, 4000])
def test_long_shared_prompt(T):
    """Two samples of one long prompt: the shared part is cut into eight pieces of 256 (2,000
    tokens) or 512 tokens (4,000 tokens), next to the rows' own split: nine partial slots,
    two batches of the merge.  Against the oracle."""
    import torch
    from oracle import decoder
    from paper_2505_24298_amd import binding
    cfg = synth.shape("tiny", n_layers=1, n_q_heads=6, n_kv_heads=1, head_dim=128, hidden=256, ffn=512,
                      rope_theta=1.0e6)
    w = synth.random_gains(synth.make_weights(cfg, 17, qkv_bias=True, std=0.03), 5)
    rng = np.random.default_rng(T)
    long_p = rng.integers(0, cfg["vocab"], size=T).astype(np.int32)
    short_p = rng.integers(0, cfg["vocab"], size=50).astype(np.int32)
    by_seq = [long_p, short_p, long_p]
    forced = rng.integers(0, cfg["vocab"], size=(2, 3)).astype(np.int32)
    w16 = _f16_weights(w)
    ref = [decoder.forward(np.concatenate([p, forced[:, i]]), w16, cfg, rows=list(range(len(p) - 1, len(p) + 2)))
           for i, p in enumerate(by_seq)]
    eng = binding.Areal(cfg, max_seqs=3, max_seq_len=T + 16, max_batch_tokens=2048,
                        kv_blocks=T // 16 + 16, convert_weights=True)
    eng.load_weights(binding.weights_to_device(w, bf16=False), 0)
    got = [eng.prefill([0, 1, 2], by_seq).cpu().numpy()]
    # the arena holds the long prompt once: the second sample shares its blocks
    for t in range(2):
        got.append(eng.decode_step([0, 1, 2], torch.from_numpy(forced[t].copy()).cuda()).cpu().numpy())
    counters = eng.decode_set_counters()
    eng.close()
    worst = max(float(np.abs(got[t][i] - ref[i][t]).max()) for t in range(3) for i in range(3))
    shared = (T - 1) // 16 * 16        # a sample computes at least its prompt's last position itself
    assert counters == (4, 4 * shared, 2 * shared)
    print(f"prompt of {T} tokens, two samples: logits {worst:.2e}", flush=True)
    assert worst <= LOGIT_TOL


def test_more_slots_than_a_row_has_every_row_walks_its_own_blocks():
    """Two sequences of 3,400 tokens that hold their first 18 blocks together, under 128-token
    splits: 25 splits of their own plus 5 shared pieces fit the 32 slots of a row, which they
    do not once the sequences are 3,750 tokens long (28 + 5 > 32).  The
    K/V are whatever the arena holds (no oracle): the logits must agree with those of the same
    launch with the sets switched off, and the counters say which way each step went."""
    import torch
    from paper_2505_24298_amd import binding
    cfg = synth.shape("tiny", n_layers=1, n_q_heads=6, n_kv_heads=1, head_dim=128, hidden=256, ffn=512,
                      rope_theta=1.0e6)
    w = binding.weights_to_device(synth.make_weights(cfg, 3, qkv_bias=True, std=0.03), bf16=False)
    saved = {k: os.environ.get(k) for k in ("AREAL_DECODE_SPLIT_TARGET", "AREAL_DECODE_MIN_CHUNK",
                                            "AREAL_DECODE_GROUPS")}
    os.environ["AREAL_DECODE_SPLIT_TARGET"] = "65536"
    os.environ["AREAL_DECODE_MIN_CHUNK"] = "128"
    out = {}
    try:
        for length, expect_rows in ((3400, 2), (3750, 0)):
            for groups_on in (True, False):
                os.environ["AREAL_DECODE_GROUPS"] = "1" if groups_on else "0"
                eng = binding.Areal(cfg, max_seqs=2, max_seq_len=length + 16, max_batch_tokens=256,
                                    kv_blocks=2 * (length // 16 + 4), convert_weights=True)
                eng.load_weights(w, 0)
                g = torch.Generator(device="cuda").manual_seed(5)
                eng.kv_arena.view(torch.float16).copy_(
                    torch.randn(eng.kv_arena.numel() // 2, generator=g, device="cuda") * 0.5)
                eng.adopt_seq(0, length, 1)
                eng.adopt_seq(1, length, 1, src_id=0, n_shared_blocks=18)
                logits = eng.decode_step([0, 1], torch.tensor([3, 4], dtype=torch.int32, device="cuda")).cpu().numpy()
                rows = eng.decode_set_counters()[0]
                eng.close()
                assert rows == (expect_rows if groups_on else 0)
                out[(length, groups_on)] = logits
            diff = float(np.abs(out[(length, True)] - out[(length, False)]).max())
            print(f"{length} tokens: sets on against off {diff:.2e}", flush=True)
            assert np.isfinite(out[(length, True)]).all() and diff <= 2e-3
    finally:
        for k, v in saved.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v
