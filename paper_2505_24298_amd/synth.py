"""Seeded synthetic inputs: model shapes, weights, prompts, output lengths.

This module only *generates inputs*.  It holds none of the method's
arithmetic and is the one module that both the CPU oracle's tests and the
GPU path's tests draw from, so that both sides see identical data.

The paper's rollouts (Section 7.1, Table 3) are math / code prompts answered
16 times each at temperature 1, top-p 1, with long and highly variable
outputs; its datasets and trained checkpoints are not available here, so the
generators below reproduce the *shape* of that workload: random-init weights
of the Qwen2 shapes, uniform random prompt tokens, prompt lengths uniform in a
range, 16 copies of every prompt, and log-normal output lengths with a cap.
"""
from __future__ import annotations

import numpy as np

SHAPES = {
    # 2-layer toy used for exhaustive parity and oracle invariants
    "tiny": dict(n_layers=2, hidden=128, n_q_heads=4, n_kv_heads=2, head_dim=32,
                 ffn=344, vocab=1024, rope_theta=1.0e4, rms_eps=1.0e-6),
    "qwen2-1.5b": dict(n_layers=28, hidden=1536, n_q_heads=12, n_kv_heads=2, head_dim=128,
                       ffn=8960, vocab=151936, rope_theta=1.0e6, rms_eps=1.0e-6),
    "qwen2-7b": dict(n_layers=28, hidden=3584, n_q_heads=28, n_kv_heads=4, head_dim=128,
                     ffn=18944, vocab=152064, rope_theta=1.0e6, rms_eps=1.0e-6),
}


def shape(name, **overrides):
    cfg = dict(SHAPES[name])
    cfg.update(overrides)
    return cfg


# ------------------------------------------------------------------ bf16 ---
def bf16_bits(x):
    """float32 array -> uint16 bf16 bit patterns, round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x):
    """float32 array rounded to the nearest bf16-representable float32."""
    return bf16_to_f32(bf16_bits(x)).reshape(np.shape(x))


# --------------------------------------------------------------- weights ---
_MATS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


def _mat_shapes(cfg):
    H, F = cfg["hidden"], cfg["ffn"]
    qd = cfg["n_q_heads"] * cfg["head_dim"]
    kd = cfg["n_kv_heads"] * cfg["head_dim"]
    return dict(wq=(qd, H), wk=(kd, H), wv=(kd, H), wo=(H, qd),
                wgate=(F, H), wup=(F, H), wdown=(H, F))


def make_weights(cfg, seed, round_bf16=False, qkv_bias=False, std=0.02):
    """Random-init parameter set as float32 numpy arrays.

    Matrices and embeddings ~ N(0, std); norm gains = 1.  Layout is
    out-features major (y = x @ W.T).  With `round_bf16` every value is
    rounded to the nearest bf16 so a bf16 device copy is exact."""
    rng = np.random.default_rng(seed)
    V, H = cfg["vocab"], cfg["hidden"]
    fix = bf16_round if round_bf16 else (lambda a: a)

    def mat(shp):
        return fix((rng.standard_normal(shp, dtype=np.float32) * np.float32(std)))

    w = dict(embed=mat((V, H)), layers=[])
    shapes = _mat_shapes(cfg)
    for _ in range(cfg["n_layers"]):
        lw = {k: mat(shapes[k]) for k in _MATS}
        lw["norm_attn"] = np.ones(H, dtype=np.float32)
        lw["norm_ffn"] = np.ones(H, dtype=np.float32)
        if qkv_bias:
            lw["bq"] = mat((shapes["wq"][0],))
            lw["bk"] = mat((shapes["wk"][0],))
            lw["bv"] = mat((shapes["wv"][0],))
        w["layers"].append(lw)
    w["final_norm"] = np.ones(H, dtype=np.float32)
    w["lm_head"] = mat((V, H))
    return w


def perturb_weights(w, seed, scale=1.0e-3, round_bf16=True, gains=False):
    """New parameter set = old + scale * N(0,1) on every matrix and embedding
    (the "fresh seeded perturbation of all weights" of the interrupt workload).
    With `gains` the norm gains move too."""
    rng = np.random.default_rng(seed)
    fix = bf16_round if round_bf16 else (lambda a: a)

    def bump(a):
        return fix(a + rng.standard_normal(a.shape, dtype=np.float32) * np.float32(scale))

    def gain(a):
        return bump(a) if gains else a.copy()

    out = dict(embed=bump(w["embed"]), layers=[])
    for lw in w["layers"]:
        nl = {}
        for k, a in lw.items():
            nl[k] = gain(a) if k.startswith("norm") else bump(a)
        out["layers"].append(nl)
    out["final_norm"] = gain(w["final_norm"])
    out["lm_head"] = bump(w["lm_head"])
    return out


def random_gains(w, seed, spread=0.2):
    """Copy of `w` whose norm gains are 1 + spread * U(-1,1): used by tests so
    that a dropped or misplaced gain shows."""
    rng = np.random.default_rng(seed)
    out = dict(w)
    out["layers"] = []
    H = w["final_norm"].shape[0]

    def g():
        return (1.0 + spread * rng.uniform(-1, 1, H)).astype(np.float32)

    for lw in w["layers"]:
        nl = dict(lw)
        nl["norm_attn"], nl["norm_ffn"] = g(), g()
        out["layers"].append(nl)
    out["final_norm"] = g()
    return out


# -------------------------------------------------------------- workload ---
def make_prompts(cfg, n_prompts, samples_per_prompt, len_lo, len_hi, seed):
    """`n_prompts` distinct prompts (length uniform in [len_lo, len_hi], tokens
    uniform over the vocabulary), each repeated `samples_per_prompt` times.
    Returns a list of int32 arrays, copies of one prompt adjacent."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n_prompts):
        n = int(rng.integers(len_lo, len_hi + 1))
        p = rng.integers(0, cfg["vocab"], size=n, dtype=np.int64).astype(np.int32)
        out.extend([p.copy() for _ in range(samples_per_prompt)])
    return out


def output_lengths(n, median, sigma, cap, seed):
    """Log-normal output lengths clip(round(exp(N(ln median, sigma))), 1, cap)."""
    rng = np.random.default_rng(seed)
    x = np.exp(rng.normal(np.log(median), sigma, size=n))
    return np.clip(np.rint(x), 1, cap).astype(np.int64)


WORKLOADS = {
    # name: shape, prompts x samples, prompt length range, output length law
    "tiny": dict(shape="tiny", n_prompts=8, samples=1, len_lo=8, len_hi=32,
                 out_fixed=64, temperature=1.0, top_p=1.0, seed=0),
    "qwen2-1.5b-rollout": dict(shape="qwen2-1.5b", n_prompts=16, samples=16, len_lo=64,
                               len_hi=512, out_median=2048, out_sigma=1.0, out_cap=8192,
                               temperature=1.0, top_p=1.0, seed=0),
    "qwen2-7b-rollout": dict(shape="qwen2-7b", n_prompts=8, samples=16, len_lo=64,
                             len_hi=512, out_median=4096, out_sigma=1.0, out_cap=16384,
                             temperature=1.0, top_p=1.0, seed=0),
    "qwen2-7b-deep": dict(shape="qwen2-7b", n_prompts=64, samples=1, len_lo=1024,
                          len_hi=1024, out_fixed=32768, temperature=0.6, top_p=0.95, seed=0),
}


def make_workload(name, scale_out=1.0):
    """Prompts and per-sequence output lengths of a named workload."""
    wl = dict(WORKLOADS[name])
    cfg = shape(wl["shape"])
    prompts = make_prompts(cfg, wl["n_prompts"], wl["samples"], wl["len_lo"], wl["len_hi"],
                           wl["seed"] + 1)
    n = len(prompts)
    if "out_fixed" in wl:
        outs = np.full(n, wl["out_fixed"], dtype=np.int64)
    else:
        outs = output_lengths(n, wl["out_median"], wl["out_sigma"], wl["out_cap"], wl["seed"] + 2)
    if scale_out != 1.0:
        outs = np.maximum(1, np.rint(outs * scale_out)).astype(np.int64)
    return cfg, wl, prompts, outs
