"""Host-side rollout loops over the C boundary (callers of the library, not
part of it): the fixed-batch rollout of the benchmark workload, the streaming
regime with the staleness gate (Sections 4.1 and 5.1 of the paper), the
on-device random-init parameter sets they run on, and the algorithmic byte and
flop counts their results are priced with.  Every forward pass, sampling step
and weight update inside these loops is one call of include/areal.h."""
from __future__ import annotations

import time

import numpy as np


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
               decode_bytes=0.0, ctx_tokens=0, ctx_tokens_distinct=0, reprefill_tokens=0, interrupts=0,
               reprefill_ms=0.0)
    # samples of one prompt hold the prompt's full KV blocks together (all but the block with the
    # last prompt token): positions that exist once in HBM however many live samples read them
    keys = {}
    group = np.array([keys.setdefault(np.asarray(p, dtype=np.int32).tobytes(), len(keys)) for p in prompts])
    shared_len = np.array([((len(p) - 1) // 16) * 16 for p in prompts])

    def distinct_ctx(live_n, gen_n):
        g = group[:live_n]
        first = np.zeros(live_n, dtype=bool)
        first[np.unique(g, return_index=True)[1]] = True
        return int((plen[:live_n] + gen_n).sum() - shared_len[:live_n][~first].sum())

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
            # in-flight weight update: the token just sampled joins its sequence first (tagged
            # with the old version, whose logits it came from; no forward pass), then every
            # prefix, that token included, is recomputed under the new weights
            a, b = ev(), ev()
            version += 1
            a.record()
            eng.append_tokens(ids[:live], toks[:live])
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
        res["ctx_tokens_distinct"] += distinct_ctx(live, gen)
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
    nxt = finished = version = steps = ticks = interrupts = retok_total = 0
    req = np.zeros(0, dtype=np.int64)          # request index of each live row
    v_sub = np.zeros(0, dtype=np.int64)        # version loaded when the request was submitted
    records = []                               # (request, version at submission, version at completion)
    gen_tokens = 0
    rows_sum = 0
    ev = lambda: torch.cuda.Event(enable_timing=True)
    e0, e1 = ev(), ev()
    torch.cuda.synchronize()
    e0.record()

    def admit(n_have):
        nonlocal nxt, ids, pos, remaining, req, v_sub
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
        req = np.concatenate([req, np.arange(nxt, nxt + k, dtype=np.int64)])
        v_sub = np.concatenate([v_sub, np.full(k, version, dtype=np.int64)])
        nxt += k

    admit(0)
    while finished < n_total:
        n = len(ids)
        assert n > 0, "gate closed with nothing in flight"
        eng.sample_logprob(logits[:n], ids, pos, temperature, top_p, seed, out=(toks[:n], lb[:n], lf[:n]))
        gen_tokens += n
        ticks += 1
        remaining -= 1
        keep = remaining > 0
        tk = toks[:n]
        if not keep.all():
            for row in sorted(np.nonzero(~keep)[0], key=lambda r: req[r]):     # in request order
                eng.free_seq(int(ids[row]))
                free_ids.append(int(ids[row]))
                finished += 1
                # the trainer steps the moment a batch is complete: later finishers of the same
                # tick already count as completed under the next version
                records.append((int(req[row]), int(v_sub[row]), (finished - 1) // train_batch))
            tk = tk[torch.from_numpy(np.nonzero(keep)[0]).to(dev)]      # row compaction (bookkeeping)
            ids, pos, remaining, req, v_sub = ids[keep], pos[keep], remaining[keep], req[keep], v_sub[keep]
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
                req, v_sub = req[order], v_sub[order]
                logits, logits_b = logits_b, logits
        admit(n_keep)
    e1.record()
    torch.cuda.synchronize()
    lib.areal_gate_destroy(gate)
    return dict(total_ms=e0.elapsed_time(e1), gen_tokens=gen_tokens, decode_steps=steps, ticks=ticks,
                records=records,
                mean_rows=rows_sum / max(steps, 1), interrupts=interrupts, reprefill_tokens=retok_total)
