"""Oracle: the decoder-only policy pi_theta(a_t | q, a_<t)  (test infrastructure).

The paper (Section 2 "LLM Training and Inference", Section 3.1) fixes only
that the policy is a dense decoder-only transformer of the Qwen2 family whose
action is one vocabulary token and whose state is the prompt followed by the
tokens generated so far, s_{t+1} = concat(s_t, a_t).  The layer arithmetic
below is the reading this build takes of that family: pre-norm blocks with
RMSNorm, grouped-query causal attention with rotary position embedding in the
rotate-half pairing, a SwiGLU feed-forward, and an untied output projection.

Everything is float64 numpy.  Weights arrive as numpy arrays (any float dtype)
in "out-features major" layout, y = x @ W.T:

    embed [V,H]  lm_head [V,H]  final_norm [H]
    layers[l]: wq [nq*d,H] wk [nkv*d,H] wv [nkv*d,H] wo [H,nq*d]
               wgate [F,H] wup [F,H] wdown [H,F] norm_attn [H] norm_ffn [H]
               optional bq [nq*d] bk [nkv*d] bv [nkv*d]

The plain definition of "logits at position t" is `next_logits`: run the whole
dense causal forward over tokens[0..t] and take the last row.  `forward`
returns all rows of one pass; `IncrementalDecoder` keeps K and V and exists
to prove that a KV cache changes nothing.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _f64(a):
    return np.asarray(a, dtype=F64)


def rmsnorm(x, g, eps):
    """y = x / sqrt(mean_j x_j^2 + eps) * g over the last axis."""
    x = _f64(x)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * _f64(g)


def rope(x, pos, theta):
    """Rotary embedding, rotate-half pairing.

    x [T, n_heads, d]; pos [T] absolute positions (first token = 0).  Pair
    (j, j + d/2) is rotated by the angle pos * theta**(-2j/d), j in [0, d/2).
    """
    x = _f64(x)
    d = x.shape[-1]
    half = d // 2
    j = np.arange(half, dtype=F64)
    freq = theta ** (-2.0 * j / d)
    ang = _f64(pos)[:, None] * freq[None, :]            # [T, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    x1 = x[..., :half]
    x2 = x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax_rows(s):
    """Softmax over the last axis."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def causal_attention(q, k, v, q_pos=None):
    """Grouped-query causal attention.

    q [Tq, nq, d]; k, v [Tk, nkv, d].  Query row i sits at absolute position
    q_pos[i] (default: i, with Tq == Tk) and sees keys j <= q_pos[i].  Query
    head a reads kv head a // (nq // nkv).  Scores are scaled by 1/sqrt(d).
    Returns [Tq, nq, d].
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    Tq, nq, d = q.shape
    Tk, nkv, _ = k.shape
    group = nq // nkv
    if q_pos is None:
        q_pos = np.arange(Tq)
    q_pos = np.asarray(q_pos)
    visible = np.arange(Tk)[None, :] <= q_pos[:, None]  # [Tq, Tk]
    out = np.empty_like(q)
    for a in range(nq):
        kv = a // group
        s = q[:, a, :] @ k[:, kv, :].T / np.sqrt(F64(d))
        s = np.where(visible, s, -np.inf)
        p = softmax_rows(s)
        out[:, a, :] = p @ v[:, kv, :]
    return out


def silu(z):
    return z / (1.0 + np.exp(-z))


def swiglu_ffn(u, wgate, wup, wdown):
    """(silu(u Wgate^T) * (u Wup^T)) Wdown^T."""
    u = _f64(u)
    return (silu(u @ _f64(wgate).T) * (u @ _f64(wup).T)) @ _f64(wdown).T


def _qkv(u, lw, cfg, pos):
    nq, nkv, d = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    q = u @ _f64(lw["wq"]).T
    k = u @ _f64(lw["wk"]).T
    v = u @ _f64(lw["wv"]).T
    if lw.get("bq") is not None:
        q = q + _f64(lw["bq"])
        k = k + _f64(lw["bk"])
        v = v + _f64(lw["bv"])
    T = u.shape[0]
    q = rope(q.reshape(T, nq, d), pos, cfg["rope_theta"])
    k = rope(k.reshape(T, nkv, d), pos, cfg["rope_theta"])
    v = v.reshape(T, nkv, d)
    return q, k, v


def hidden_states(tokens, w, cfg):
    """Residual stream after the last block, one dense causal pass, [T, H]."""
    tokens = np.asarray(tokens, dtype=np.int64)
    T = tokens.shape[0]
    pos = np.arange(T)
    eps = cfg["rms_eps"]
    h = _f64(w["embed"][tokens])
    for lw in w["layers"]:
        u = rmsnorm(h, lw["norm_attn"], eps)
        q, k, v = _qkv(u, lw, cfg, pos)
        o = causal_attention(q, k, v)
        h = h + o.reshape(T, -1) @ _f64(lw["wo"]).T
        u = rmsnorm(h, lw["norm_ffn"], eps)
        h = h + swiglu_ffn(u, lw["wgate"], lw["wup"], lw["wdown"])
    return h


def logits_from_hidden(h, w, cfg):
    return rmsnorm(h, w["final_norm"], cfg["rms_eps"]) @ _f64(w["lm_head"]).T


def forward(tokens, w, cfg, rows=None):
    """Logits of one dense causal pass over `tokens`; row t = logits for the
    token that follows tokens[0..t].  `rows` restricts the output projection
    to those positions (the layer stack still runs over every position)."""
    h = hidden_states(tokens, w, cfg)
    if rows is not None:
        h = h[np.asarray(rows)]
    return logits_from_hidden(h, w, cfg)


def next_logits(tokens, w, cfg):
    """The plain definition: logits for the next token given the whole prefix,
    recomputed from scratch with no cache."""
    return forward(tokens, w, cfg, rows=[len(tokens) - 1])[0]


class IncrementalDecoder:
    """One sequence decoded token by token with stored K and V.  Exists to
    show that caching keys and values reproduces the plain definition."""

    def __init__(self, w, cfg):
        self.w, self.cfg = w, cfg
        L = cfg["n_layers"]
        self.k = [[] for _ in range(L)]
        self.v = [[] for _ in range(L)]
        self.n = 0

    def reset_cache(self):
        for l in range(self.cfg["n_layers"]):
            self.k[l].clear()
            self.v[l].clear()
        self.n = 0

    def append(self, tokens):
        """Feed one or more new tokens; return the logits after the last."""
        tokens = np.atleast_1d(np.asarray(tokens, dtype=np.int64))
        cfg, w = self.cfg, self.w
        T = tokens.shape[0]
        pos = np.arange(self.n, self.n + T)
        eps = cfg["rms_eps"]
        h = _f64(w["embed"][tokens])
        for l, lw in enumerate(w["layers"]):
            u = rmsnorm(h, lw["norm_attn"], eps)
            q, k, v = _qkv(u, lw, cfg, pos)
            self.k[l].extend(k)
            self.v[l].extend(v)
            o = causal_attention(q, np.stack(self.k[l]), np.stack(self.v[l]), q_pos=pos)
            h = h + o.reshape(T, -1) @ _f64(lw["wo"]).T
            u = rmsnorm(h, lw["norm_ffn"], eps)
            h = h + swiglu_ffn(u, lw["wgate"], lw["wup"], lw["wdown"])
        self.n += T
        return logits_from_hidden(h[-1:], w, cfg)[0]
