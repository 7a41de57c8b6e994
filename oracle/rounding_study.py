"""Rounding study (test infrastructure; calls only oracle/ and the input generators).

Re-runs the float64 oracle forward pass with the values that the GPU path
stores in 16 bits (normalised activations `xn`, rotated q and k, v, softmax
probabilities `p`, attention output `attn`, SwiGLU output `act`) rounded to a
16-bit format, one group at a time, and reports the logit error each group
alone causes at the Qwen2-1.5B shape with N(0, 0.02) weights.  This is the
arithmetic behind the choice of half precision (fp16) over bf16 for matrix
operands and K/V:  python -m oracle.rounding_study [bf16|fp16]
"""
import sys, time
import numpy as np
from oracle import decoder as D
from paper_2505_24298_amd import synth

FMT = sys.argv[1] if len(sys.argv) > 1 else "bf16"


def r(x):
    """Round to the nearest value of the 16-bit format under study."""
    x32 = np.asarray(x, dtype=np.float32)
    if FMT == "fp16":
        return x32.astype(np.float16).astype(np.float64)
    return synth.bf16_round(x32).astype(np.float64)

def forward_emul(tokens, w, cfg, which):
    T = len(tokens); pos = np.arange(T); eps = cfg["rms_eps"]
    nq, nkv, d = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    h = D._f64(w["embed"][tokens])
    R = lambda name, x: r(x) if name in which else x
    for lw in w["layers"]:
        u = R("xn", D.rmsnorm(h, lw["norm_attn"], eps))
        q = (u @ D._f64(lw["wq"]).T).astype(np.float32).astype(np.float64)
        k = (u @ D._f64(lw["wk"]).T).astype(np.float32).astype(np.float64)
        v = (u @ D._f64(lw["wv"]).T).astype(np.float32).astype(np.float64)
        q = R("q", D.rope(q.reshape(T, nq, d), pos, cfg["rope_theta"]))
        k = R("k", D.rope(k.reshape(T, nkv, d), pos, cfg["rope_theta"]))
        v = R("v", v.reshape(T, nkv, d))
        # attention with optional P rounding
        out = np.empty_like(q)
        vis = np.arange(T)[None, :] <= pos[:, None]
        for a in range(nq):
            kv = a // (nq // nkv)
            s = q[:, a] @ k[:, kv].T / np.sqrt(d)
            s = np.where(vis, s, -np.inf)
            m = s.max(-1, keepdims=True)
            e = np.exp(s - m)
            l = e.sum(-1, keepdims=True)
            out[:, a] = (R("p", e) @ v[:, kv]) / l
        o = R("attn", out.reshape(T, -1))
        h = h + o @ D._f64(lw["wo"]).T
        u = R("xn", D.rmsnorm(h, lw["norm_ffn"], eps))
        g = u @ D._f64(lw["wgate"]).T
        up = u @ D._f64(lw["wup"]).T
        act = R("act", D.silu(g) * up)
        h = h + act @ D._f64(lw["wdown"]).T
    x = R("xn", D.rmsnorm(h[-8:], w["final_norm"], eps))
    return x @ D._f64(w["lm_head"]).T

cfg = synth.shape("qwen2-1.5b")
t0 = time.time()
w = synth.make_weights(cfg, 0, round_bf16=True)
print("weights", time.time() - t0, flush=True)
toks = np.random.default_rng(1).integers(0, cfg["vocab"], 96)
ref = forward_emul(toks, w, cfg, set())
print("ref done", time.time() - t0, "logit std", ref.std(), flush=True)
print("format", FMT)
for which in [{"xn", "q", "k", "v", "p", "attn", "act"}, {"xn"}, {"act"}, {"attn"}, {"p"}, {"q"}, {"k"}, {"v"}, {"k", "v"}]:
    got = forward_emul(toks, w, cfg, which)
    err = got - ref
    print(sorted(which), "rms err", err.std(), "max", np.abs(err).max(), "rel", err.std() / ref.std(), flush=True)
