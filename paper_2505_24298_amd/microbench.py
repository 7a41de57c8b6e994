#!/usr/bin/env python3
"""Single-kernel microbenchmarks on the MI355X (tuning and profiling aids).

  python3 paper_2505_24298_amd/microbench.py attn-decode [shared [steps,...]]
      decode steps at the context mixes the qwen2-1.5b-rollout workload has after
      500 / 1500 / 3000 / 5000 / 7000 generated tokens (sequences adopted at those
      lengths, K/V pool filled with N(0,1)); reports the decode-attention launch
      time and bandwidth (HIP events inside the library) and the step time.  With
      `shared` the samples of a prompt hold the prompt's KV blocks together, as after
      areal_prefill of the workload (16 samples per prompt), and the line also gives
      the distinct context tokens per launch.
  python3 paper_2505_24298_amd/microbench.py gemm-chosen [M,M,...] [shape,...] [working set in MB]
      the projection GEMMs at the library's own tile choice only (a short run for
      rocprofv3 --pmc: bytes fetched against weight bytes, matrix-core busy cycles).
      The weights rotate over 1.2 GB (every launch reads them from HBM) or over the
      given working set (150: they sit in the 256 MB memory-side cache, in no L2).
  python3 paper_2505_24298_amd/microbench.py gemm [M,M,...] [shape,...]
      every tile configuration x K split of the projection GEMM at the decoder's
      shapes (qkv, o, gateup, down, lmhead of the 1.5B shape; qkv7 ... lmhead7 of the 7B shape);
      weights rotate over
      > 1 GB so they come from HBM.
  python3 paper_2505_24298_amd/microbench.py read
      what a kernel that only reads reaches per launch size (32 MiB .. 1 GiB), each launch
      between its own pair of events: the yardstick for the decode attention launch.
  python3 paper_2505_24298_amd/microbench.py copy
      four plain 1 GiB device-to-device copies: the calibration of the FETCH_SIZE /
      WRITE_SIZE counters (known bytes per dispatch).
  python3 paper_2505_24298_amd/microbench.py prefill [qwen2-1.5b|qwen2-7b]
      prefill of 32x256, 8x2048, 4x8000 tokens: per-kernel time of one layer.
  python3 paper_2505_24298_amd/microbench.py score
      teacher-forced log-prob pass over 64 trajectories of 512..4096 tokens at the
      1.5B shape, output projection over 256 / 1024 / 4096 rows at a time.
"""
from __future__ import annotations

import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np


def _weights(torch, cfg):
    from paper_2505_24298_amd.harness import device_weights
    return device_weights(torch, cfg, 0, "cuda:0")


def attn_decode(shared=False, steps=(500, 1500, 3000, 5000, 7000)):
    import torch
    from paper_2505_24298_amd import binding, synth
    cfg, wl, prompts, outs = synth.make_workload("qwen2-1.5b-rollout")
    w = _weights(torch, cfg)
    kvb = 2 * cfg["n_kv_heads"] * cfg["head_dim"] * 2
    group = wl["samples"]
    for step in steps:
        live = [i for i, o in enumerate(outs) if o > step]
        lens = [len(prompts[i]) + step for i in live]
        B = len(lens)
        eng = binding.Areal(cfg, max_seqs=B, max_seq_len=max(lens) + 64, max_batch_tokens=max(B, 256),
                            kv_blocks=sum(l // 16 + 6 for l in lens))
        eng.load_weights(w, 0)
        eng.kv_arena.view(torch.float16).normal_()
        leader, distinct = {}, 0
        for s, (i, l) in enumerate(zip(live, lens)):
            g = i // group
            n_sh = (len(prompts[i]) - 1) // 16
            if shared and g in leader and n_sh > 0:
                eng.adopt_seq(s, l, 1, src_id=leader[g], n_shared_blocks=n_sh)
                distinct += l - 16 * n_sh
            else:
                eng.adopt_seq(s, l, 1)
                leader.setdefault(g, s)
                distinct += l
        ids = np.arange(B, dtype=np.int32)
        toks = torch.ones(B, dtype=torch.int32, device="cuda")
        for _ in range(3):
            eng.decode_step(ids, toks)
        eng.profile_begin(binding.K_ATTN_DECODE, 0, 1)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n = 12
        e0.record()
        for _ in range(n):
            eng.decode_step(ids, toks)
        e1.record()
        cnt, ms, units = eng.profile_end()
        print(json.dumps(dict(after_tokens=step, sequences=B, mean_context=int(np.mean(lens)),
                              context_tokens_per_launch=int(units / cnt),
                              distinct_context_tokens_per_launch=int(distinct + 3 * B + (n + 1) * B / 2),
                              attn_launch_us=round(ms / cnt * 1e3, 2),
                              attn_GBps=round(units * kvb / (ms * 1e-3) / 1e9, 1),
                              step_ms=round(e0.elapsed_time(e1) / n, 3))), flush=True)
        eng.close()
        del eng


def read_calibration():
    import torch
    from paper_2505_24298_amd import binding
    total = 3 << 30
    buf = torch.empty(total, dtype=torch.uint8, device="cuda")
    buf.view(torch.int32).random_()
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    off = 0
    for mb in (32, 64, 128, 192, 256, 512, 1024):
        n = mb << 20
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(14)]
        for a, b in ev:
            if off + n > total:
                off = 0
            a.record()
            binding.op_stream_read(buf, off, n, sink)
            b.record()
            off += n
        torch.cuda.synchronize()
        us = [a.elapsed_time(b) * 1e3 for a, b in ev[2:]]
        print(json.dumps(dict(read_MiB=mb, launches=len(us), us=round(sum(us) / len(us), 2),
                              GBps=round(n / (sum(us) / len(us) * 1e-6) / 1e9, 1))), flush=True)


def copy_calibration():
    import torch
    a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()
    b = torch.empty_like(a)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    b.copy_(a)
    e0.record()
    for _ in range(3):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    print(json.dumps(dict(copies=4, bytes_each=1 << 30, GBps_read_plus_write=round(3 * 2 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1))))


def gemm_chosen(ms_arg, shapes_arg, iters=20, working_set=1.2e9):
    import torch
    from paper_2505_24298_amd import binding
    g = torch.Generator(device="cuda").manual_seed(0)
    for name in shapes_arg.split(","):
        N, K, mode = GEMM_SHAPES[name]
        wbytes = N * K * 2 * (2 if mode == 2 else 1)
        # weights rotate over `working_set` bytes: > 1 GB = every launch reads them from HBM; 150 MB = they
        # were read a few launches ago and sit in the memory-side cache (256 MB) but in no L2 (8 x 4 MB)
        ncopy = max(2, min(64, int(working_set // wbytes)))
        mk = lambda: (torch.randn((N, K), generator=g, device="cuda") * 0.02).to(torch.float16)
        Ws = [mk() for _ in range(ncopy)]
        W1s = [mk() for _ in range(ncopy)] if mode == 2 else None
        for M in [int(x) for x in ms_arg.split(",")]:
            As = [torch.randn((M, K), generator=g, device="cuda").to(torch.float16) for _ in range(ncopy)]
            Cs = [torch.zeros((M, N), device="cuda", dtype=torch.float16 if mode == 2 else torch.float32)
                  for _ in range(ncopy)]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for it in range(2 * iters):
                if it == iters:
                    e0.record()
                i = it % ncopy
                binding.op_gemm(As[i], Ws[i], None if W1s is None else W1s[i], Cs[i], mode, -1,
                                1 if name.startswith("lmhead") else -1)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / iters
            print(json.dumps(dict(shape=name, M=M, launches=2 * iters, us=round(us, 2), weight_bytes=wbytes,
                                  a_bytes=M * K * 2, weight_GBps=round(wbytes / us / 1e3, 1),
                                  TFLOPs=round(2.0 * M * N * K * (2 if mode == 2 else 1) / us / 1e6, 1))), flush=True)
            del As, Cs
        del Ws, W1s


GEMM_SHAPES = {"qkv": (2048, 1536, 0), "o": (1536, 1536, 1), "gateup": (8960, 1536, 2),
               "down": (1536, 8960, 1), "lmhead": (151936, 1536, 0),
               # the 7B shape
               "qkv7": (4608, 3584, 0), "o7": (3584, 3584, 1), "gateup7": (18944, 3584, 2),
               "down7": (3584, 18944, 1), "lmhead7": (152064, 3584, 0)}


def gemm(ms_arg, shapes_arg):
    import torch
    from paper_2505_24298_amd import binding
    L = binding.lib()
    ncfg = L.areal_op_gemm_num_configs()
    shapes = GEMM_SHAPES
    Ms = [int(x) for x in ms_arg.split(",")]
    g = torch.Generator(device="cuda").manual_seed(0)
    for name in shapes_arg.split(","):
        N, K, mode = shapes[name]
        wbytes = N * K * 2 * (2 if mode == 2 else 1)
        ncopy = max(2, min(64, int(1.2e9 // wbytes)))
        mk = lambda: (torch.randn((N, K), generator=g, device="cuda") * 0.02).to(torch.float16)
        Ws = [mk() for _ in range(ncopy)]
        W1s = [mk() for _ in range(ncopy)] if mode == 2 else None
        for M in Ms:
            # A and C rotate too: inside a decode step both were last touched by another kernel
            # (on other XCDs), never by the previous launch of this product
            As = [torch.randn((M, K), generator=g, device="cuda").to(torch.float16) for _ in range(ncopy)]
            Cs = [torch.zeros((M, N), device="cuda", dtype=torch.float16 if mode == 2 else torch.float32)
                  for _ in range(ncopy)]
            for cfg in range(ncfg):
                for splits in ([1] if mode == 2 or name.startswith("lmhead") else [1, 2, 3, 4, 6, 8, 12]):
                    if cfg >= 7 and K % 64:
                        continue
                    iters = 3 * ncopy if wbytes < 1e8 else 6

                    def run(n):
                        for i in range(n):
                            binding.op_gemm(As[i % ncopy], Ws[i % ncopy], None if W1s is None else W1s[i % ncopy],
                                            Cs[i % ncopy], mode, cfg, splits)
                    try:
                        run(ncopy if wbytes < 1e8 else 2)
                    except binding.ArealError:        # configuration does not serve this epilogue
                        continue
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    run(iters)
                    e1.record()
                    torch.cuda.synchronize()
                    us = e0.elapsed_time(e1) * 1e3 / iters
                    print(json.dumps(dict(shape=name, M=M, cfg=cfg, splits=splits, us=round(us, 2),
                                          weight_GBps=round(wbytes / us / 1e3, 1),
                                          TFLOPs=round(2.0 * M * N * K * (2 if mode == 2 else 1) / us / 1e6, 1))),
                          flush=True)
            del As, Cs
        del Ws, W1s


def prefill(shape_name="qwen2-1.5b"):
    import torch
    from paper_2505_24298_amd import binding, synth
    cfg = synth.shape(shape_name)
    w = _weights(torch, cfg)
    classes = [(binding.K_ATTN_PREFILL, "attn"), (binding.K_GEMM_GATEUP, "gateup"), (binding.K_GEMM_DOWN, "down"),
               (binding.K_GEMM_QKV, "qkv"), (binding.K_GEMM_O, "o")]
    for n_seq, plen in [(32, 256), (8, 2048), (4, 8000)]:
        eng = binding.Areal(cfg, max_seqs=n_seq, max_seq_len=plen + 8, max_batch_tokens=8192,
                            kv_blocks=n_seq * (plen // 16 + 2))
        eng.load_weights(w, 0)
        prompts = synth.make_prompts(cfg, n_seq, 1, plen, plen, seed=3)
        ids = list(range(n_seq))
        eng.prefill(ids, prompts)                     # untimed: loads the code objects
        for s in ids:
            eng.free_seq(s)
        res = dict(sequences=n_seq, prompt_len=plen)
        for klass, nm in classes:
            eng.profile_begin(klass, 0, 1)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            eng.prefill(ids, prompts)
            e1.record()
            cnt, ms, units = eng.profile_end()
            res[nm + "_ms_layer0"] = round(ms, 3)
            if nm == "attn":
                res["attn_TFLOPs"] = round(units * 4 * cfg["n_q_heads"] * cfg["head_dim"] / (ms * 1e-3) / 1e12, 1)
            total = e0.elapsed_time(e1)
            for s in ids:
                eng.free_seq(s)
        res.update(total_ms=round(total, 1), tokens_per_s=round(n_seq * plen / total * 1e3))
        print(json.dumps(res), flush=True)
        eng.close()
        del eng


def score():
    import torch
    from paper_2505_24298_amd import binding, synth
    cfg = synth.shape("qwen2-1.5b")
    w = _weights(torch, cfg)
    rng = np.random.default_rng(4)
    lens = rng.integers(512, 4097, size=64)
    seqs = [rng.integers(0, cfg["vocab"], size=int(n)).astype(np.int32) for n in lens]
    total = int(lens.sum())
    eng = binding.Areal(cfg, max_seqs=64, max_seq_len=4096, max_batch_tokens=8192, kv_blocks=total // 16 + 128)
    eng.load_weights(w, 0)
    flops_tok = 2.0 * (1543656960 - 0)          # all matrices incl. the output projection, per token
    attn = 4.0 * cfg["n_q_heads"] * cfg["head_dim"] * cfg["n_layers"] * float((lens * (lens + 1) / 2).sum())
    for rows in (256, 1024, 4096):
        scratch = torch.empty((rows, cfg["vocab"]), dtype=torch.float32, device="cuda")
        eng.recompute_logprob(seqs[:2], 1.0, scratch=scratch)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        out = eng.recompute_logprob(seqs, 1.0, scratch=scratch)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        print(json.dumps(dict(sequences=64, tokens=total, scratch_rows=rows, ms=round(ms, 1),
                              tokens_per_s=round(total / ms * 1e3),
                              TFLOPs=round((flops_tok * total + attn) / (ms * 1e-3) / 1e12, 1),
                              mean_logp=round(float(out.mean()), 3))), flush=True)
        del scratch
    eng.close()


if __name__ == "__main__":
    what = sys.argv[1] if len(sys.argv) > 1 else ""
    if what == "attn-decode":
        if len(sys.argv) > 3:
            attn_decode(shared=sys.argv[2] == "shared", steps=tuple(int(x) for x in sys.argv[3].split(",")))
        else:
            attn_decode(shared=len(sys.argv) > 2 and sys.argv[2] == "shared")
    elif what == "copy":
        copy_calibration()
    elif what == "read":
        read_calibration()
    elif what == "gemm-chosen":
        gemm_chosen(sys.argv[2] if len(sys.argv) > 2 else "24,100,256",
                    sys.argv[3] if len(sys.argv) > 3 else "qkv,o,gateup,down,lmhead",
                    working_set=float(sys.argv[4]) * 1e6 if len(sys.argv) > 4 else 1.2e9)
    elif what == "gemm":
        gemm(sys.argv[2] if len(sys.argv) > 2 else "32,64,128,256",
             sys.argv[3] if len(sys.argv) > 3 else "qkv,o,gateup,down,lmhead")
    elif what == "prefill":
        prefill(sys.argv[2] if len(sys.argv) > 2 else "qwen2-1.5b")
    elif what == "score":
        score()
    else:
        print(__doc__)
        sys.exit(2)
