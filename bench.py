#!/usr/bin/env python3
"""Benchmark of the rollout hot path on one MI355X.

One "step" = one whole rollout of the named workload: prefill of every
prompt, then sample + decode until every sequence has produced its pre-drawn
number of tokens (weights and prompts resident in HBM before the clock
starts).  With --interrupt-every N the in-flight weight update of the paper's
interruptible rollout fires every N decode steps (new weights prepared
beforehand), as in the interrupt workload.

A rollout of the headline workload takes tens of seconds, so the run works to
an all-in wall-clock budget (--budget-s, counted from process start: imports,
weight initialisation, the CPU leg, warm-up and the timed rollouts).  Warm-up
steps are rollouts with every output length scaled down (--warmup-scale); of the
--steps timed rollouts asked for, as many run as the budget allows (at least one),
and the JSON line reports that number as `steps`.  Progress goes to stderr
after every rollout; SIGTERM prints the line for the rollouts completed so far.

Prints ONE JSON line on stdout: generated tokens/s for the whole job, the
roofline of the dominant kernel (paged decode attention, HBM-bound) measured
with HIP events inside the timed region, and the CPU oracle timed on the host
cores as a baseline.
"""
from __future__ import annotations

import time

T_PROCESS_START = time.perf_counter()

import argparse
import json
import os
import signal
import sys

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_F16_PEAK_TFLOPS = 2500.0   # MI355X published dense fp16 / bf16
SHAPE_LABEL = {"qwen2-1.5b": "Qwen2-1.5B", "qwen2-7b": "Qwen2-7B", "tiny": "tiny"}
# HBM bytes the decode attention kernel moves, from rocprofv3 FETCH_SIZE / WRITE_SIZE runs
# calibrated with a plain copy (profiles/attn_decode_kernel_hbm_traffic.md): bytes fetched per
# byte of K/V that exists once in HBM (the samples of a prompt read the same prompt blocks; a
# block is fetched about once per launch), and bytes written per per-sequence K/V byte read
ATTN_DECODE_FETCH_OVER_DISTINCT = 1.033
ATTN_DECODE_WRITE_OVER_ALGORITHMIC = 0.028


def log(msg):
    print(f"[bench {time.perf_counter() - T_PROCESS_START:7.1f}s] {msg}", file=sys.stderr, flush=True)


def measured_copy_bandwidth(torch, dev, gib=2, reps=5):
    """Bytes read + written per second by a plain device-to-device copy of `gib` GiB
    (what this machine's HBM sustains for a trivially simple kernel), in GB/s."""
    n = gib << 30
    a = torch.empty(n, dtype=torch.uint8, device=dev)
    b = torch.empty(n, dtype=torch.uint8, device=dev)
    a.zero_()
    b.copy_(a)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    del a, b
    torch.cuda.empty_cache()
    return 2.0 * n / (ms * 1e-3) / 1e9


def measured_read_bandwidth(torch, binding, dev, sizes_mb=(32, 64, 128, 256, 512), reps=12):
    """What a kernel that only reads reaches on this machine, per launch size: [(bytes, GB/s)], each launch
    between its own pair of events (as the library brackets the attention launch), over a 2 GiB buffer
    walked in order so that no launch finds its bytes in a cache."""
    total = 2 << 30
    buf = torch.empty(total, dtype=torch.uint8, device=dev)
    buf.view(torch.int32).random_()
    sink = torch.zeros(16, dtype=torch.uint8, device=dev)
    out = []
    off = 0
    for mb in sizes_mb:
        n = mb << 20
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            if off + n > total:
                off = 0
            a.record()
            binding.op_stream_read(buf, off, n, sink)
            b.record()
            off += n
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in ev[2:])
        out.append((n, n / (sum(ms) / len(ms) * 1e-3) / 1e9))
    del buf
    torch.cuda.empty_cache()
    return out


def read_bandwidth_at(curve, nbytes):
    """GB/s of a plain read of nbytes, interpolated (in launch time) between the measured sizes."""
    pts = [(b, b / (g * 1e9)) for b, g in curve]                 # (bytes, seconds)
    if nbytes <= pts[0][0]:
        t = pts[0][1] * nbytes / pts[0][0]
    elif nbytes >= pts[-1][0]:
        t = pts[-1][1] * nbytes / pts[-1][0]
    else:
        for (b0, t0), (b1, t1) in zip(pts, pts[1:]):
            if b0 <= nbytes <= b1:
                t = t0 + (t1 - t0) * (nbytes - b0) / (b1 - b0)
                break
    return nbytes / t / 1e9


def cpu_oracle_baseline(cfg_name, host_weights, budget_s=20.0):
    """The CPU oracle as it stands (incremental-KV variant, numpy float64) on a
    bounded slice of the same workload: 4 sequences of the workload's model
    shape, prompts cut to 32 tokens, decode steps until the time budget is
    reached, one weight update (an interrupt: K/V dropped, every prefix
    recomputed) after the second step.  Returns generated tokens/s over the
    decode steps of that slice; the prefill and the interrupt are reported
    beside it."""
    import threadpoolctl
    from oracle import rollout as orollout
    from paper_2505_24298_amd import synth
    cfg = synth.shape(cfg_name)
    n_seq = 4
    prompts = synth.make_prompts(cfg, n_seq, 1, 32, 32, seed=1)
    ids = list(range(n_seq))
    wk = orollout.RolloutWorker(cfg, host_weights, version=0, seed=0, use_cache=True)
    t0 = time.perf_counter()
    for s, p in zip(ids, prompts):
        wk.add(s, p)
    t_prefill = time.perf_counter() - t0
    steps, t_dec, t_int = 0, 0.0, 0.0
    while True:
        t1 = time.perf_counter()
        wk.step(ids)
        t_dec += time.perf_counter() - t1
        steps += 1
        if steps == 2:
            t1 = time.perf_counter()
            wk.update_weights(host_weights, 1)
            t_int = time.perf_counter() - t1
        if steps >= 32 or (steps >= 2 and time.perf_counter() - t0 > budget_s):
            break
    threads = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
    return dict(value=round(n_seq * steps / t_dec, 3), unit="gen tokens/s", cores=int(threads),
                nproc=os.cpu_count(), kind="oracle",
                sample=f"{cfg_name} shape, {n_seq} sequences x 32-token prompts, {steps} decode steps "
                       f"({n_seq * steps} tokens in {t_dec:.1f} s), one weight update + re-prefill of all "
                       f"prefixes after step 2 ({t_int:.1f} s), prefill of the {n_seq * 32} prompt tokens "
                       f"{t_prefill:.1f} s; incremental-KV float64 numpy oracle; the rate counts decode steps only")


def host_copy_of(w):
    """Device parameter set -> the same values as float32 numpy arrays (the oracle's input)."""
    cv = lambda t: t.float().cpu().numpy()
    return dict(embed=cv(w["embed"]), lm_head=cv(w["lm_head"]), final_norm=cv(w["final_norm"]),
                layers=[{k: cv(v) for k, v in lw.items()} for lw in w["layers"]])


def depth_sweep(args):
    """Decode-step time against context depth for the deep-context workload
    (64 sequences of the 7B shape, T=0.6, top-p=0.95): the paged pool is taken
    as already holding `depth` tokens per sequence (areal_adopt_seq: no
    generation up to that depth), then --sweep-steps decode steps are timed.
    Prints one JSON line per depth; not the headline benchmark."""
    import torch
    from paper_2505_24298_amd import binding, synth
    from paper_2505_24298_amd.harness import decode_step_bytes, device_weights
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
    from paper_2505_24298_amd.harness import device_weights, rollout, streaming_rollout
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


def summarise(args, cfg, wl, n, runs, warmups_done, copy_gbs, cpu_baseline, binding, read_curve=None):
    """The JSON line for the timed rollouts in `runs`."""
    steps = len(runs)
    total_s = sum(r["total_ms"] for r in runs) / 1e3
    gen = sum(r["gen_tokens"] for r in runs)
    dec_ms = sum(r["decode_ms"] for r in runs)
    pre_ms = sum(r["prefill_ms"] for r in runs)
    dec_bytes = sum(r["decode_bytes"] for r in runs)
    dec_steps = sum(r["decode_steps"] for r in runs)
    pn, pms, punits = (sum(r["profile"][i] for r in runs) for i in range(3)) if "profile" in runs[0] else (0, 0.0, 0.0)
    kv_layer_bytes = 2 * cfg["n_kv_heads"] * cfg["head_dim"] * 2          # K+V bytes per token per layer
    if args.profile_class == binding.K_ATTN_DECODE and pn:
        achieved = punits * kv_layer_bytes / (pms * 1e-3) / 1e9
        alg_per_launch = punits * kv_layer_bytes / pn
        # every launch of a step reads the same contexts: whole-run averages per launch
        ctx_all = sum(r["ctx_tokens"] for r in runs)
        distinct_per_launch = alg_per_launch * sum(r["ctx_tokens_distinct"] for r in runs) / max(ctx_all, 1)
        roofline = dict(bound="hbm", kernel="attn_decode_kernel", achieved=round(achieved, 1),
                        peak=HBM_PEAK_GBS, unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4),
                        traffic=int(distinct_per_launch * ATTN_DECODE_FETCH_OVER_DISTINCT
                                    + alg_per_launch * ATTN_DECODE_WRITE_OVER_ALGORITHMIC),
                        traffic_unit="bytes per launch: rocprofv3 FETCH_SIZE + WRITE_SIZE of this kernel at this "
                                     "workload's context mixes and block sharing, taken on microbench.py (the counter "
                                     "profiler does not survive bench.py) as ratios to the K/V bytes that exist once "
                                     "in HBM (fetch) and to the algorithmic bytes (write), applied to this run's bytes "
                                     "per launch (profiles/attn_decode_kernel_hbm_traffic.md)",
                        frac_of_measured_copy=None if not copy_gbs else round(achieved / copy_gbs, 4),
                        algorithmic_bytes_per_launch=int(alg_per_launch),
                        distinct_kv_bytes_per_launch=int(distinct_per_launch),
                        launches_timed=int(pn), avg_launch_us=round(pms / pn * 1e3, 2),
                        avg_context_tokens_per_launch=round(punits / pn, 1))
        if read_curve:
            # the same bytes through a kernel that only reads them, bracketed the same way
            rd = read_bandwidth_at(read_curve, roofline["traffic"])
            roofline["plain_read_GBps_at_traffic"] = round(rd, 1)
            roofline["launch_time_of_plain_read_over_kernel"] = round(
                (roofline["traffic"] / (rd * 1e9)) / (pms / pn * 1e-3), 4)
            roofline["plain_read_curve"] = [[int(b), round(g, 1)] for b, g in read_curve]
    else:
        roofline = dict(bound="hbm", kernel=f"class {args.profile_class}", achieved=None, peak=HBM_PEAK_GBS,
                        unit="GB/s", frac=None, traffic=None, launches_timed=int(pn),
                        avg_launch_us=round(pms / max(pn, 1) * 1e3, 2))
    dec_gbs = dec_bytes / (dec_ms * 1e-3) / 1e9
    out = {
        "metric": f"gen tokens/s, 1 MI355X, {SHAPE_LABEL.get(wl['shape'], wl['shape'])} shape; decode HBM GB/s % of peak",
        "value": round(gen / total_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": steps,
        "warmup": warmups_done, "ms_per_step": round(total_s * 1e3 / steps, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": args.workload + (f" x{args.scale_out} output length" if args.scale_out != 1 else "")
                   + (f", weight update every {args.interrupt_every} decode steps" if args.interrupt_every else ""),
                   "sequences": n, "prompt_tokens": runs[0]["prefill_tokens"],
                   "generated_tokens": runs[0]["gen_tokens"], "decode_steps": runs[0]["decode_steps"],
                   "sampling": f"T={wl['temperature']} top_p={wl['top_p']}",
                   "steps_requested": args.steps, "warmup_requested": args.warmup,
                   "step": "one whole rollout; warm-up steps are rollouts at "
                           f"x{args.warmup_scale} output length; timed steps capped by --budget-s {args.budget_s:g}"},
        "decode": {"tokens_per_s": round(gen / (dec_ms * 1e-3), 1),
                   "hbm_GBps_algorithmic": round(dec_gbs, 1),
                   "hbm_frac_of_peak": round(dec_gbs / HBM_PEAK_GBS, 4),
                   "hbm_frac_of_measured_copy": None if not copy_gbs else round(dec_gbs / copy_gbs, 4),
                   "measured_copy_GBps": None if not copy_gbs else round(copy_gbs, 1),
                   # against a kernel that only reads, at the largest launch size measured (512 MiB)
                   "hbm_frac_of_plain_read": None if not read_curve else round(dec_gbs / read_curve[-1][1], 4),
                   "ms_per_decode_step": round(dec_ms / max(1, dec_steps), 4),
                   "attn_decode_launches": cfg["n_layers"] * dec_steps,
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
    if cpu_baseline is not None:
        out["cpu_baseline"] = cpu_baseline
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--budget-s", type=float, default=360.0,
                    help="all-in wall-clock budget from process start; the timed rollouts stop when the next "
                         "one would not fit (at least one runs)")
    ap.add_argument("--warmup-scale", type=float, default=0.05,
                    help="output-length scale of the warm-up rollouts")
    ap.add_argument("--workload", default="qwen2-1.5b-rollout")
    ap.add_argument("--scale-out", type=float, default=1.0, help="scale every output length (quick runs)")
    ap.add_argument("--interrupt-every", type=int, default=0)
    ap.add_argument("--max-batch-tokens", type=int, default=8192)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget-s", type=float, default=20.0)
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
    if args.steps < 1 or args.warmup < 0:
        print("bench.py: --steps must be >= 1 and --warmup >= 0", file=sys.stderr)
        sys.exit(2)

    log("importing torch")
    import torch
    from paper_2505_24298_amd import binding, synth
    from paper_2505_24298_amd.harness import device_weights, rollout
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
    log(f"workload {args.workload}: {n} sequences, {int(np.sum(out_lens))} tokens to generate")
    w0 = device_weights(torch, cfg, 0, dev)
    weight_sets = [w0]
    if args.interrupt_every:
        weight_sets.append(device_weights(torch, cfg, 1001, dev, base=w0, scale=1e-3))
    torch.cuda.synchronize()
    log("weights initialised")

    cpu_baseline = None
    if not args.no_cpu_baseline:
        hw = host_copy_of(w0)
        cpu_baseline = cpu_oracle_baseline(wl["shape"], hw, args.cpu_budget_s)
        del hw
        log(f"cpu oracle: {cpu_baseline['value']} tokens/s")
    copy_gbs = measured_copy_bandwidth(torch, dev)
    log(f"device copy: {copy_gbs:.0f} GB/s read+write")
    read_curve = measured_read_bandwidth(torch, binding, dev)
    log("plain read: " + ", ".join(f"{b >> 20} MiB {g:.0f} GB/s" for b, g in read_curve))

    eng = binding.Areal(cfg, max_seqs=n, max_seq_len=max_len, max_batch_tokens=args.max_batch_tokens,
                        kv_blocks=kv_blocks)
    # priming run (untimed, not a warm-up step): 2 sequences, 3 tokens: loads the code objects
    eng.load_weights(w0, 0)
    rollout(eng, torch, cfg, prompts[:2], [3, 3], wl["temperature"], wl["top_p"], 0)

    runs, warmups_done = [], 0
    state = dict(printed=False)

    def emit():
        if state["printed"] or not runs:
            return
        state["printed"] = True
        print(json.dumps(summarise(args, cfg, wl, n, runs, warmups_done, copy_gbs, cpu_baseline, binding,
                                   read_curve)), flush=True)

    def on_term(signum, frame):
        log(f"signal {signum}: reporting the {len(runs)} rollouts completed")
        emit()
        os._exit(0 if runs else 1)

    signal.signal(signal.SIGTERM, on_term)

    def one_rollout(lens, profile):
        eng.load_weights(w0, 0)
        return rollout(eng, torch, cfg, prompts, lens, wl["temperature"], wl["top_p"], 0,
                       interrupt_every=args.interrupt_every, weight_sets=weight_sets, profile=profile)

    left = lambda: args.budget_s - (time.perf_counter() - T_PROCESS_START)
    warm_lens = np.maximum(1, np.rint(np.asarray(out_lens) * args.warmup_scale)).astype(np.int64)
    est = None                                       # seconds per full rollout
    for it in range(args.warmup):
        t0 = time.perf_counter()
        r = one_rollout(warm_lens, None)
        dt = time.perf_counter() - t0
        warmups_done += 1
        # a full rollout costs more than 1/scale warm-ups' decode steps (contexts grow): first guess only
        est = max(est or 0.0, dt / max(args.warmup_scale, 1e-3) * 0.6)
        log(f"warm-up {it + 1}/{args.warmup}: {r['gen_tokens']} tokens in {dt:.2f} s")
        if left() < 3 * dt + (est or 0.0):
            break
    prof = (args.profile_class, 0, args.profile_every) if args.profile_class >= 0 else None
    for it in range(args.steps):
        if runs and left() < 1.15 * est + 5.0:
            log(f"budget: {left():.0f} s left, next rollout needs ~{est:.0f} s: stopping after {len(runs)} of "
                f"{args.steps} timed rollouts")
            break
        t0 = time.perf_counter()
        r = one_rollout(out_lens, prof)
        dt = time.perf_counter() - t0
        est = dt
        runs.append(r)
        log(f"rollout {it + 1}/{args.steps}: {r['gen_tokens']} tokens in {r['total_ms'] / 1e3:.2f} s = "
            f"{r['gen_tokens'] / (r['total_ms'] * 1e-3):.0f} tokens/s, decode "
            f"{r['decode_ms'] / max(1, r['decode_steps']):.3f} ms/step")
    eng.close()
    emit()


if __name__ == "__main__":
    main()
