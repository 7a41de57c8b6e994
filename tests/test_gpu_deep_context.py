"""GPU parity at head_dim 128 and the context depths the timed workloads reach:
prompts of up to 8,150 tokens prefilled in chunks (several attention tiles and
several passes per sequence), then forced decode steps over sequences of mixed
depth (64 .. 8,150 tokens) in one launch, with the KV walk cut in as many as 32
splits, in splits longer than 64 blocks, and in the default partition; query
groups of 6 (the 1.5B geometry, one and two KV heads) and 7 (the 7B geometry).
Few layers and a narrow residual stream keep the float64 oracle affordable; the
attention kernels see the full head geometry.  Logits against the oracle's plain
full-sequence forward, same tolerance as everywhere: 2e-2."""
import os

import numpy as np
import pytest

from paper_2505_24298_amd import synth

pytestmark = pytest.mark.gpu

LOGIT_TOL = 2e-2
DEEP = [64, 700, 2100, 8150]
MID = [64, 700, 4100]               # two layers and two KV heads at an affordable oracle cost
N_DECODE = 3


def _f16(a):
    return np.asarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)


def _f16_weights(w):
    return dict(embed=_f16(w["embed"]), lm_head=_f16(w["lm_head"]), final_norm=_f16(w["final_norm"]),
                layers=[{k: _f16(v) for k, v in lw.items()} for lw in w["layers"]])


# (split target, minimum split length) -> partition of the deepest sequence (8,150 .. 8,153 tokens;
# 4,100 .. 4,103 in the two-layer case: 17 splits of 256, or 3 of 2,048):
#   (65536, 128): splits of 256 tokens, 32 of them (the limit);
#   (64, 2048):   splits of 2,048 tokens = 128 blocks (both halves of the per-lane block-id pair);
#   (None, None): the library's own choice
KNOBS = [(65536, 128), (64, 2048), (None, None)]


@pytest.mark.parametrize("nq,nkv,layers,DEPTHS", [(6, 1, 1, DEEP), (7, 1, 1, DEEP), (12, 2, 2, MID)])
def test_head_dim_128_deep_mixed_contexts(nq, nkv, layers, DEPTHS):
    import torch
    from oracle import decoder
    from paper_2505_24298_amd import binding
    cfg = synth.shape("tiny", n_layers=layers, n_q_heads=nq, n_kv_heads=nkv, head_dim=128, hidden=256,
                      ffn=512, rope_theta=1.0e6)
    w = synth.random_gains(synth.make_weights(cfg, 70 + nq, qkv_bias=True, std=0.03), 9)
    rng = np.random.default_rng(100 + nq)
    prompts = [rng.integers(0, cfg["vocab"], size=T).astype(np.int32) for T in DEPTHS]
    forced = rng.integers(0, cfg["vocab"], size=(N_DECODE, len(DEPTHS))).astype(np.int32)
    w16 = _f16_weights(w)
    ref = []                                     # per sequence: rows T-1 .. T-1+N_DECODE
    for i, p in enumerate(prompts):
        seq = np.concatenate([p, forced[:, i]])
        T = len(p)
        ref.append(decoder.forward(seq, w16, cfg, rows=list(range(T - 1, T + N_DECODE))))
    ids = list(range(len(prompts)))
    saved = {k: os.environ.get(k) for k in ("AREAL_DECODE_SPLIT_TARGET", "AREAL_DECODE_MIN_CHUNK")}
    try:
        for target, min_chunk in KNOBS:
            for k, v in (("AREAL_DECODE_SPLIT_TARGET", target), ("AREAL_DECODE_MIN_CHUNK", min_chunk)):
                if v is None:
                    os.environ.pop(k, None)
                else:
                    os.environ[k] = str(v)
            print(f"heads {nq}/{nkv}, split target {target}, min chunk {min_chunk}", flush=True)
            eng = binding.Areal(cfg, max_seqs=len(ids), max_seq_len=max(DEPTHS) + N_DECODE + 8,
                                max_batch_tokens=2048, kv_blocks=sum(T // 16 + 2 for T in DEPTHS),
                                convert_weights=True)
            eng.load_weights(binding.weights_to_device(w, bf16=False), 0)
            got = [eng.prefill(ids, prompts).cpu().numpy()]
            for t in range(N_DECODE):
                got.append(eng.decode_step(ids, torch.from_numpy(forced[t].copy()).cuda()).cpu().numpy())
            eng.close()
            worst = 0.0
            for i in ids:
                for t in range(N_DECODE + 1):
                    worst = max(worst, float(np.abs(got[t][i] - ref[i][t]).max()))
            print(f"  logits {worst:.2e}", flush=True)
            assert worst <= LOGIT_TOL
    finally:
        for k, v in saved.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v
