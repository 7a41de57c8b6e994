#!/usr/bin/env python3
"""Benchmark of the rollout hot path on one MI355X.

One "step" = one whole rollout of the named workload: prefill of every
prompt, then sample + decode until every sequence has produced its pre-drawn
number of tokens (weights and prompts resident in HBM before the clock
starts).  With --interrupt-every N the in-flight weight update of the paper's
interruptible rollout fires every N decode steps (new weights prepared
beforehand), as in the interrupt workload.

Prints ONE JSON line: generated tokens/s for the whole job, the roofline of the
dominant kernel (paged decode attention, HBM-bound) measured with HIP events
inside the timed region, and the CPU oracle timed on the host cores as a
baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_F16_PEAK_TFLOPS = 2500.0   # MI355X published dense fp16 / bf16
SHAPE_LABEL = {"qwen2-1.5b": "Qwen2-1.5B", "qwen2-7b": "Qwen2-7B", "tiny": "tiny"}
# HBM bytes the decode attention kernel moves per algorithmic K/V byte, from rocprofv3
# FETCH_SIZE / WRITE_SIZE runs calibrated with a plain copy (profiles/attn_decode_kernel_hbm_traffic.md)
ATTN_DECODE_FETCH_OVER_ALGORITHMIC = 1.024
ATTN_DECODE_WRITE_OVER_ALGORITHMIC = 0.028


def device_weights(torch, cfg, seed, device, base=None, scale=None):
    """Random-init bf16 parameter set on the device: matrices and embeddings
    N(0, 0.02), gains 1.  With `base`: base + scale * N(0,1) (the interrupt
    workload's perturbed weights).  The library converts a bf16 set to its
    half-precision operand format when it receives it."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)

    def mat(shape, old=None):
        x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        if old is None:
            x.mul_(0.02)
        else:
            x.mul_(scale).add_(old.float())
        return x.to(torch.bfloat16).contiguous()

    H, F, V = cfg["hidden"], cfg["ffn"], cfg["vocab"]
    qd, kd = cfg["n_q_heads"] * cfg["head_dim"], cfg["n_kv_heads"] * cfg["head_dim"]
    shapes = dict(wq=(qd, H), wk=(kd, H), wv=(kd, H), wo=(H, qd), wgate=(F, H), wup=(F, H), wdown=(H, F))
    ones = lambda: torch.ones(H, device=device, dtype=torch.bfloat16)
    w = dict(embed=mat((V, H), None if base is None else base["embed"]), layers=[])
    for l in range(cfg["n_layers"]):
        lw = {k: mat(s, None if base is None else base["layers"][l][k]) for k, s in shapes.items()}
        lw["norm_attn"], lw["norm_ffn"] = ones(), ones()
        w["layers"].append(lw)
    w["final_norm"] = ones()
    w["lm_head"] = mat((V, H), None if base is None else base["lm_head"])
    return w


def decode_step_bytes(cfg, ctx_sum, n):
    """Algorithmic HBM bytes of one decode step over n sequences whose contexts
    sum to ctx_sum tokens: every weight once, every cached K/V once, the new K/V
    rows, the logits written once and read once by the sampler."""
    H, F, V, L = cfg["hidden"], cfg["ffn"], cfg["vocab"], cfg["n_layers"]
    qd, kd = cfg["n_q_heads"] * cfg["head_dim"], cfg["n_kv_heads"] * cfg["head_dim"]
    w_elems = L * (qd * H + 2 * kd * H + H * qd + 3 * F * H + 2 * H) + H + V * H
    kv_token = L * 2 * kd * 2
    return 2 * w_elems + kv_token * ctx_sum + kv_token * n + 2 * 4 * n * V


def prefill_work(cfg, prompts):
    """Rows and flops the library really computes for one areal_prefill call over
    `prompts`: a prompt equal to an earlier one of the call shares that one's full
    KV blocks (all but the block holding the last token) and computes only the
    positions after them."""
    H, F, V, L = cfg["hidden"], cfg["ffn"], cfg["vocab"], cfg["n_layers"]
    qd, kd = cfg["n_q_heads"] * cfg["head_dim"], cfg["n_kv_heads"] * cfg["head_dim"]
    p_layers = L * (qd * H + 2 * kd * H + H * qd + 3 * F * H)
    seen = set()
    rows, pairs = 0, 0.0
    for p in prompts:
        key = np.asarray(p, dtype=np.int32).tobytes()
        n = len(p)
        start = ((n - 1) // 16) * 16 if key in seen else 0
        seen.add(key)
        rows += n - start
        pairs += n * (n + 1) / 2 - start * (start + 1) / 2
    return rows, float(2 * p_layers * rows + 2 * V * H * len(prompts) + 4 * qd * L * pairs)


def reprefill_flops(cfg, prompts, lens, retok):
    """Flops of one re-prefill over live sequences of the given current lengths:
    a prompt's shared blocks are recomputed by the first live sequence holding
    them only (retok = positions the library reports as recomputed)."""
    H, F, V, L = cfg["hidden"], cfg["ffn"], cfg["vocab"], cfg["n_layers"]
    qd, kd = cfg["n_q_heads"] * cfg["head_dim"], cfg["n_kv_heads"] * cfg["head_dim"]
    p_layers = L * (qd * H + 2 * kd * H + H * qd + 3 * F * H)
    seen, pairs, rows = set(), 0.0, 0
    for p, n in zip(prompts, lens):
        key = np.asarray(p, dtype=np.int32).tobytes()
        start = ((len(p) - 1) // 16) * 16 if key in seen else 0
        seen.add(key)
        n = int(n)
        rows += n - start
        pairs += n * (n + 1) / 2 - start * (start + 1) / 2
    assert rows == retok, (rows, retok)
    return float(2 * p_layers * rows + 2 * V * H * len(prompts) + 4 * qd * L * pairs)


def rollout(eng, torch, cfg, prompts, out_lens, temperature, top_p, seed, interrupt_every=0,
            weight_sets=None, profile=None):
    """Run one whole rollout.  Sequences are ordered by output length
    (longest first) so the live set is always a prefix of the batch.  Returns
    timings and counters."""
    order = np.argsort(-np.asarray(out_lens), kind="stable")
    prompts = [prompts[i] for i in order]
    out_lens = np.asarray(out_lens)[order]
    n = len(prompts)
    ids = np.arange(n, dtype=np.int32)
    plen = np.array([len(p) for p in prompts])
    dev = eng.device
    logits = torch.empty((n, cfg["vocab"]), dtype=torch.float32, device=dev)
    logits_b = torch.empty_like(logits) if interrupt_every else None
    toks = torch.empty(n, dtype=torch.int32, device=dev)
    lb = torch.empty(n, dtype=torch.float32, device=dev)
    lf = torch.empty(n, dtype=torch.float32, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    e_start, e_prefill, e_end = ev(), ev(), ev()
    res = dict(prefill_tokens=int(plen.sum()), gen_tokens=int(out_lens.sum()), decode_steps=0,
               decode_bytes=0.0, ctx_tokens=0, reprefill_tokens=0, interrupts=0, reprefill_ms=0.0)
    re_events = []

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e_start.record()
    eng.prefill(ids, prompts, logits_out=logits)
    e_prefill.record()
    if profile is not None:
        eng.profile_begin(profile[0], profile[1], profile[2])
    gen = 0                                     # tokens generated so far per live sequence
    live = n
    max_new = int(out_lens.max())
    version = 0
    while True:
        # sample token number gen+1 for every live sequence
        eng.sample_logprob(logits[:live], ids[:live], plen[:live] + gen, temperature, top_p, seed,
                           out=(toks[:live], lb[:live], lf[:live]))
        gen += 1
        # sequences whose output is complete leave (they sit at the tail of the order)
        new_live = int(np.searchsorted(-out_lens, -gen, side="left"))      # out_lens > gen
        for s in range(new_live, live):
            eng.free_seq(s)
        live = new_live
        if live == 0:
            break
        if interrupt_every and gen % interrupt_every == 0:
            # in-flight weight update: the token just sampled is appended first (its
            # logits came from the old version), then every prefix is recomputed
            a, b = ev(), ev()
            eng.decode_step(ids[:live], toks[:live], logits_out=logits[:live])
            res["decode_bytes"] += decode_step_bytes(cfg, int((plen[:live] + gen).sum()), live)
            res["ctx_tokens"] += int((plen[:live] + gen).sum())
            res["decode_steps"] += 1
            version += 1
            a.record()
            _, _, retok = eng.update_weights_interrupt(weight_sets[version % len(weight_sets)], version,
                                                       logits_out=logits_b)
            b.record()
            res["reprefill_flops"] = res.get("reprefill_flops", 0.0) + reprefill_flops(
                cfg, prompts[:live], plen[:live] + gen, retok)
            re_events.append((a, b))
            logits, logits_b = logits_b, logits
            res["reprefill_tokens"] += retok
            res["interrupts"] += 1
            continue
        eng.decode_step(ids[:live], toks[:live], logits_out=logits[:live])
        res["decode_bytes"] += decode_step_bytes(cfg, int((plen[:live] + gen).sum()), live)
        res["ctx_tokens"] += int((plen[:live] + gen).sum())
        res["decode_steps"] += 1
    e_end.record()
    torch.cuda.synchronize()
    res["wall_s"] = time.perf_counter() - t0
    if profile is not None:
        res["profile"] = eng.profile_end()
    res["total_ms"] = e_start.elapsed_time(e_end)
    res["prefill_ms"] = e_start.elapsed_time(e_prefill)
    res["reprefill_ms"] = float(sum(a.elapsed_time(b) for a, b in re_events))
    res["decode_ms"] = res["total_ms"] - res["prefill_ms"] - res["reprefill_ms"]
    res["prefill_rows"], res["prefill_flops"] = prefill_work(cfg, prompts)
    res["max_new"] = max_new
    return res


def streaming_rollout(eng, torch, cfg, lib, prompts, out_lens, slots, train_batch, eta, weight_sets,
                      temperature, top_p, seed):
    """The paper's streaming regime on one GPU (Sections 4.1, 5.1): `slots`
    sequences decode together; a finished sequence's slot is refilled with the
    next prompt as long as the staleness gate floor((N_r-1)/B) <= i + eta admits
    it; every `train_batch` finished trajectories the (simulated) trainer
    publishes a new version, which interrupts the generation in flight
    (areal_update_weights_interrupt: all prefixes recomputed).  eta = 0 is the
    synchronous schedule.  Returns timings and counters."""
    n_total = len(prompts)
    dev = eng.device
    V = cfg["vocab"]
    logits = torch.empty((slots, V), dtype=torch.float32, device=dev)
    logits_b = torch.empty_like(logits)
    toks = torch.empty(slots, dtype=torch.int32, device=dev)
    lb = torch.empty(slots, dtype=torch.float32, device=dev)
    lf = torch.empty(slots, dtype=torch.float32, device=dev)
    gate = lib.areal_gate_create(train_batch, eta)
    free_ids = list(range(slots - 1, -1, -1))
    ids = np.zeros(0, dtype=np.int32)          # live sequences, row order
    pos = np.zeros(0, dtype=np.int64)          # current length = position of the next token
    remaining = np.zeros(0, dtype=np.int64)
    nxt = finished = version = steps = interrupts = retok_total = 0
    gen_tokens = 0
    rows_sum = 0
    ev = lambda: torch.cuda.Event(enable_timing=True)
    e0, e1 = ev(), ev()
    torch.cuda.synchronize()
    e0.record()

    def admit(n_have):
        nonlocal nxt, ids, pos, remaining
        want = min(len(free_ids), n_total - nxt)
        k = int(lib.areal_gate_submit(gate, want)) if want > 0 else 0
        if k == 0:
            return
        new_ids = [free_ids.pop() for _ in range(k)]
        new_prompts = prompts[nxt:nxt + k]
        eng.prefill(new_ids, new_prompts, logits_out=logits[n_have:n_have + k])
        ids = np.concatenate([ids, np.asarray(new_ids, dtype=np.int32)])
        pos = np.concatenate([pos, np.asarray([len(p) for p in new_prompts], dtype=np.int64)])
        remaining = np.concatenate([remaining, np.asarray(out_lens[nxt:nxt + k], dtype=np.int64)])
        nxt += k

    admit(0)
    while finished < n_total:
        n = len(ids)
        assert n > 0, "gate closed with nothing in flight"
        eng.sample_logprob(logits[:n], ids, pos, temperature, top_p, seed, out=(toks[:n], lb[:n], lf[:n]))
        gen_tokens += n
        remaining -= 1
        keep = remaining > 0
        tk = toks[:n]
        if not keep.all():
            for s in ids[~keep]:
                eng.free_seq(int(s))
                free_ids.append(int(s))
            finished += int((~keep).sum())
            tk = tk[torch.from_numpy(np.nonzero(keep)[0]).to(dev)]      # row compaction (bookkeeping)
            ids, pos, remaining = ids[keep], pos[keep], remaining[keep]
        n_keep = len(ids)
        if n_keep:
            eng.decode_step(ids, tk.contiguous(), logits_out=logits[:n_keep])
            pos = pos + 1
            steps += 1
            rows_sum += n_keep
        if finished // train_batch > version:                 # the trainer has stepped
            version = finished // train_batch
            lib.areal_gate_set_version(gate, version)
            live, _, retok = eng.update_weights_interrupt(weight_sets[version % len(weight_sets)], version,
                                                          logits_out=logits_b)
            interrupts += 1
            retok_total += retok
            if len(live):                                     # logits now come in ascending id order
                order = np.argsort(ids, kind="stable")
                assert ids[order].tolist() == live.tolist()
                ids, pos, remaining = ids[order], pos[order], remaining[order]
                logits, logits_b = logits_b, logits
        admit(n_keep)
    e1.record()
    torch.cuda.synchronize()
    lib.areal_gate_destroy(gate)
    return dict(total_ms=e0.elapsed_time(e1), gen_tokens=gen_tokens, decode_steps=steps,
                mean_rows=rows_sum / max(steps, 1), interrupts=interrupts, reprefill_tokens=retok_total)


def cpu_oracle_baseline(cfg_name, budget_s=20.0):
    """The CPU oracle as it stands (incremental-KV variant, numpy float64) on a
    bounded slice of the same workload: 2 sequences of the workload's model
    shape, prompts cut to 32 tokens, a few decode steps, stopping near the time
    budget.  Returns generated tokens/s over that slice."""
    import threadpoolctl
    from oracle import rollout as orollout
    from paper_2505_24298_amd import synth
    cfg = synth.shape(cfg_name)
    t_w = time.perf_counter()
    w = synth.make_weights(cfg, 0, round_bf16=True)
    t_w = time.perf_counter() - t_w
    prompts = synth.make_prompts(cfg, 2, 1, 32, 32, seed=1)
    wk = orollout.RolloutWorker(cfg, w, version=0, seed=0, use_cache=True)
    t0 = time.perf_counter()
    for s, p in enumerate(prompts):
        wk.add(s, p)
    t_prefill = time.perf_counter() - t0
    steps = 0
    t1 = time.perf_counter()
    while time.perf_counter() - t0 < budget_s or steps < 2:
        wk.step([0, 1])
        steps += 1
        if steps >= 64:
            break
    t_dec = time.perf_counter() - t1
    threads = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
    return dict(value=round(2 * steps / t_dec, 3), unit="gen tokens/s", cores=int(threads), kind="oracle",
                sample=f"{cfg_name} shape, 2 sequences x 32-token prompts, {steps} decode steps "
                       f"(incremental-KV float64 numpy oracle; prefill of the 64 prompt tokens took "
                       f"{t_prefill:.1f} s and is not in the rate)")


def depth_sweep(args):
    """Decode-step time against context depth for the deep-context workload
    (64 sequences of the 7B shape, T=0.6, top-p=0.95): the paged pool is taken
    as already holding `depth` tokens per sequence (areal_adopt_seq: no
    generation up to that depth), then --sweep-steps decode steps are timed.
    Prints one JSON line per depth; not the headline benchmark."""
    import torch
    from paper_2505_24298_amd import binding, synth
    cfg, wl, _, _ = synth.make_workload(args.workload)
    n = wl["n_prompts"] * wl["samples"]
    depths = [int(x) for x in args.depth_sweep.split(",")]
    steps = args.sweep_steps
    w0 = device_weights(torch, cfg, 0, "cuda:0")
    for depth in depths:
        eng = binding.Areal(cfg, max_seqs=n, max_seq_len=depth + steps + 8, max_batch_tokens=max(n, 256),
                            kv_blocks=n * ((depth + steps) // 16 + 2))
        eng.load_weights(w0, 0)
        eng.kv_arena.view(torch.float16).normal_()               # K/V contents: N(0,1) halves, not zeros
        for s_ in range(n):
            eng.adopt_seq(s_, depth, 1)
        ids = np.arange(n, dtype=np.int32)
        logits = torch.zeros((n, cfg["vocab"]), dtype=torch.float32, device="cuda:0")
        out = (torch.ones(n, dtype=torch.int32, device="cuda:0"), torch.empty(n, device="cuda:0"),
               torch.empty(n, device="cuda:0"))
        eng.decode_step(ids, out[0], logits_out=logits)          # untimed first step
        eng.profile_begin(binding.K_ATTN_DECODE, 0, 1)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        nbytes = 0.0
        e0.record()
        for t in range(steps):
            eng.sample_logprob(logits, ids, np.full(n, depth + 1 + t), wl["temperature"], wl["top_p"], 0, out=out)
            eng.decode_step(ids, out[0], logits_out=logits)
            nbytes += decode_step_bytes(cfg, n * (depth + 2 + t), n)
        e1.record()
        cnt, ams, units = eng.profile_end()
        ms = e0.elapsed_time(e1)
        kvb = 2 * cfg["n_kv_heads"] * cfg["head_dim"] * 2
        print(json.dumps({"workload": args.workload, "sequences": n, "depth": depth, "decode_steps": steps,
                          "ms_per_decode_step": round(ms / steps, 3), "gen_tokens_per_s": round(n * steps / ms * 1e3, 1),
                          "hbm_GBps_algorithmic": round(nbytes / (ms * 1e-3) / 1e9, 1),
                          "hbm_frac_of_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                          "attn_decode_GBps": round(units * kvb / (ams * 1e-3) / 1e9, 1),
                          "attn_decode_us": round(ams / cnt * 1e3, 1)}), flush=True)
        eng.close()
        del eng, logits, out
        torch.cuda.empty_cache()


def streaming(args):
    import torch
    from paper_2505_24298_amd import binding, synth
    dev = "cuda:0"
    wl = dict(synth.WORKLOADS[args.workload])
    cfg = synth.shape(wl["shape"])
    n_total, slots = args.streaming, wl["n_prompts"] * wl["samples"]
    assert n_total % wl["samples"] == 0
    prompts = synth.make_prompts(cfg, n_total // wl["samples"], wl["samples"], wl["len_lo"], wl["len_hi"],
                                 wl["seed"] + 1)
    outs = synth.output_lengths(n_total, wl["out_median"], wl["out_sigma"], wl["out_cap"], wl["seed"] + 2)
    if args.scale_out != 1.0:
        outs = np.maximum(1, np.rint(outs * args.scale_out)).astype(np.int64)
    max_len = wl["len_hi"] + int(outs.max()) + 1
    eng = binding.Areal(cfg, max_seqs=slots, max_seq_len=max_len, max_batch_tokens=args.max_batch_tokens,
                        kv_blocks=slots * (max_len // 16 + 2))
    w0 = device_weights(torch, cfg, 0, dev)
    weight_sets = [w0, device_weights(torch, cfg, 1001, dev, base=w0, scale=1e-3)]
    eng.load_weights(w0, 0)
    rollout(eng, torch, cfg, prompts[:2], [3, 3], wl["temperature"], wl["top_p"], 0)      # loads the code objects
    eng.load_weights(w0, 0)
    r = streaming_rollout(eng, torch, cfg, binding.lib(), prompts, outs, slots, args.train_batch, args.eta,
                          weight_sets, wl["temperature"], wl["top_p"], 0)
    out = {"metric": "gen tokens/s, 1 MI355X, streaming rollout with staleness gate", "unit": "tokens/s",
           "value": round(r["gen_tokens"] / (r["total_ms"] * 1e-3), 1), "n_gpus": 1,
           "ms_total": round(r["total_ms"], 1), "dtype": "f16", "data": "synthetic",
           "config": {"workload": args.workload + f" streamed: {n_total} trajectories through {slots} slots, "
                      f"training batch {args.train_batch}, eta {args.eta}"
                      + (f", x{args.scale_out} output length" if args.scale_out != 1 else "")},
           "generated_tokens": r["gen_tokens"], "decode_steps": r["decode_steps"],
           "mean_rows_per_step": round(r["mean_rows"], 1), "weight_updates": r["interrupts"],
           "reprefilled_tokens": r["reprefill_tokens"]}
    eng.close()
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1)
    ap.add_argument("--warmup", type=int, default=0)
    ap.add_argument("--workload", default="qwen2-1.5b-rollout")
    ap.add_argument("--scale-out", type=float, default=1.0, help="scale every output length (quick runs)")
    ap.add_argument("--interrupt-every", type=int, default=0)
    ap.add_argument("--max-batch-tokens", type=int, default=8192)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-class", type=int, default=4,
                    help="kernel class bracketed with HIP events (-1: none, e.g. under rocprofv3 --pmc)")
    ap.add_argument("--profile-every", type=int, default=16)
    ap.add_argument("--depth-sweep", default="", help="comma-separated context depths: time decode steps at "
                    "each depth (deep-context workload) instead of the rollout")
    ap.add_argument("--sweep-steps", type=int, default=32)
    ap.add_argument("--streaming", type=int, default=0, help="streaming regime: total trajectories "
                    "(multiple of 16), slots refilled as sequences finish, staleness gate, weight "
                    "update + interrupt every --train-batch finished trajectories")
    ap.add_argument("--eta", type=int, default=4, help="maximum staleness for --streaming (0 = synchronous)")
    ap.add_argument("--train-batch", type=int, default=256)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one MI355X: this build has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_24298_amd import binding, synth
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    if args.depth_sweep:
        depth_sweep(args)
        return
    if args.streaming:
        streaming(args)
        return
    dev = "cuda:0"
    cfg, wl, prompts, out_lens = synth.make_workload(args.workload, scale_out=args.scale_out)
    n = len(prompts)
    max_len = int(max(len(p) + o for p, o in zip(prompts, out_lens))) + 1
    # KV pool: what the workload can hold at its peak, plus slack
    peak_tokens = int(sum(len(p) + o for p, o in zip(prompts, out_lens)))
    kv_blocks = peak_tokens // 16 + 2 * n + 64
    eng = binding.Areal(cfg, max_seqs=n, max_seq_len=max_len, max_batch_tokens=args.max_batch_tokens,
                        kv_blocks=kv_blocks)
    w0 = device_weights(torch, cfg, 0, dev)
    weight_sets = [w0]
    if args.interrupt_every:
        weight_sets.append(device_weights(torch, cfg, 1001, dev, base=w0, scale=1e-3))
    # priming run (untimed, not a warmup step): 2 sequences, 3 tokens: loads the code objects
    eng.load_weights(w0, 0)
    rollout(eng, torch, cfg, prompts[:2], [3, 3], wl["temperature"], wl["top_p"], 0)

    runs = []
    for it in range(args.warmup + args.steps):
        eng.load_weights(w0, 0)
        prof = (args.profile_class, 0, args.profile_every) if args.profile_class >= 0 else None
        r = rollout(eng, torch, cfg, prompts, out_lens, wl["temperature"], wl["top_p"], 0,
                    interrupt_every=args.interrupt_every, weight_sets=weight_sets, profile=prof)
        if it >= args.warmup:
            runs.append(r)
    total_s = sum(r["total_ms"] for r in runs) / 1e3
    gen = sum(r["gen_tokens"] for r in runs)
    dec_ms = sum(r["decode_ms"] for r in runs)
    pre_ms = sum(r["prefill_ms"] for r in runs)
    dec_bytes = sum(r["decode_bytes"] for r in runs)
    pn, pms, punits = (sum(r["profile"][i] for r in runs) for i in range(3)) if "profile" in runs[0] else (0, 0.0, 0.0)
    kv_layer_bytes = 2 * cfg["n_kv_heads"] * cfg["head_dim"] * 2          # K+V bytes per token per layer
    if args.profile_class == binding.K_ATTN_DECODE and pn:
        achieved = punits * kv_layer_bytes / (pms * 1e-3) / 1e9
        alg_per_launch = punits * kv_layer_bytes / pn
        roofline = dict(bound="hbm", kernel="attn_decode_kernel", achieved=round(achieved, 1),
                        peak=HBM_PEAK_GBS, unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4),
                        traffic=int(alg_per_launch * (ATTN_DECODE_FETCH_OVER_ALGORITHMIC
                                                      + ATTN_DECODE_WRITE_OVER_ALGORITHMIC)),
                        traffic_unit="bytes per launch (counter ratios of profiles/attn_decode_kernel_hbm_traffic.md"
                                     " x this run's algorithmic bytes per launch)",
                        algorithmic_bytes_per_launch=int(alg_per_launch),
                        launches_timed=int(pn), avg_launch_us=round(pms / pn * 1e3, 2),
                        avg_context_tokens_per_launch=round(punits / pn, 1))
    else:
        roofline = dict(bound="hbm", kernel=f"class {args.profile_class}", achieved=None, peak=HBM_PEAK_GBS,
                        unit="GB/s", frac=None, traffic=None, launches_timed=int(pn),
                        avg_launch_us=round(pms / max(pn, 1) * 1e3, 2))
    out = {
        "metric": f"gen tokens/s, 1 MI355X, {SHAPE_LABEL.get(wl['shape'], wl['shape'])} shape; decode HBM GB/s % of peak",
        "value": round(gen / total_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(total_s * 1e3 / args.steps, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": args.workload + (f" x{args.scale_out} output length" if args.scale_out != 1 else "")
                   + (f", weight update every {args.interrupt_every} decode steps" if args.interrupt_every else ""),
                   "sequences": n, "prompt_tokens": runs[0]["prefill_tokens"],
                   "generated_tokens": runs[0]["gen_tokens"], "decode_steps": runs[0]["decode_steps"],
                   "sampling": f"T={wl['temperature']} top_p={wl['top_p']}"},
        "decode": {"tokens_per_s": round(gen / (dec_ms * 1e-3), 1),
                   "hbm_GBps_algorithmic": round(dec_bytes / (dec_ms * 1e-3) / 1e9, 1),
                   "hbm_frac_of_peak": round(dec_bytes / (dec_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                   "ms_per_decode_step": round(dec_ms / max(1, sum(r["decode_steps"] for r in runs)), 4),
                   "attn_decode_launches": cfg["n_layers"] * sum(r["decode_steps"] for r in runs),
                   "attn_decode_kv_bytes_algorithmic": int(kv_layer_bytes * cfg["n_layers"]
                                                           * sum(r["ctx_tokens"] for r in runs))},
        "prefill": {"tokens_per_s": round(sum(r["prefill_tokens"] for r in runs) / (pre_ms * 1e-3), 1),
                    "computed_tokens_per_s": round(sum(r["prefill_rows"] for r in runs) / (pre_ms * 1e-3), 1),
                    "computed_tokens": int(runs[0]["prefill_rows"]),
                    "mfma_frac_of_peak": round(sum(r["prefill_flops"] for r in runs) / (pre_ms * 1e-3)
                                               / (MFMA_F16_PEAK_TFLOPS * 1e12), 4),
                    "note": "the 16 samples of a prompt share its KV blocks: computed_tokens are the rows "
                            "that really ran; mfma_frac counts their flops only"},
        "roofline": roofline,
    }
    if args.interrupt_every:
        rt, rms = sum(r["reprefill_tokens"] for r in runs), sum(r["reprefill_ms"] for r in runs)
        out["interrupt"] = {"count": runs[0]["interrupts"], "reprefill_tokens_per_s": round(rt / (rms * 1e-3), 1),
                            "reprefill_mfma_frac_of_peak": round(sum(r["reprefill_flops"] for r in runs) / (rms * 1e-3)
                                                                 / (MFMA_F16_PEAK_TFLOPS * 1e12), 4),
                            "reprefill_ms_total": round(rms, 1),
                            "reprefill_over_decode_time": round(rms / dec_ms, 4)}
    eng.close()
    del eng
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_oracle_baseline(wl["shape"])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
