"""Oracle: token log-probabilities of whole trajectories  (test infrastructure).

Section 5.2 of the paper: the decoupled PPO objective (Eq. 5) weighs each token
by pi_theta / pi_prox and pi_prox / pi_behav.  pi_behav comes with the rollout;
the proximal policy's log-probabilities are recomputed over the complete
trajectories when a training batch has arrived, with the parameters the
trainer holds at that moment.  What is computed is the plain definition

    logp[t] = log softmax(logits(x_0 .. x_{t-1}) / T)[x_t],     t = 1 .. L-1,

with logp[0] = 0 (nothing predicts the first token).  No cache, no packing:
one dense causal forward per sequence in float64, a log-sum-exp per row and a
gather.
"""
from __future__ import annotations

import numpy as np

from . import decoder


def log_softmax_rows(z):
    """log softmax over the last axis, float64."""
    z = np.asarray(z, dtype=np.float64)
    m = z.max(axis=-1, keepdims=True)
    return z - m - np.log(np.exp(z - m).sum(axis=-1, keepdims=True))


def sequence_logprobs(tokens, w, cfg, temperature=1.0):
    """float64 [L]: log-probability of every token of `tokens` given the tokens
    before it, under the decoder with weights `w`, at sampling temperature T."""
    tokens = np.asarray(tokens, dtype=np.int64)
    L = len(tokens)
    out = np.zeros(L, dtype=np.float64)
    if L < 2:
        return out
    logits = decoder.forward(tokens[:-1], w, cfg)          # row t predicts token t+1
    lp = log_softmax_rows(logits / float(temperature))
    out[1:] = lp[np.arange(L - 1), tokens[1:]]
    return out


def batch_logprobs(seqs, w, cfg, temperature=1.0):
    """Packed float64 [sum of lengths] for a list of token sequences."""
    return np.concatenate([sequence_logprobs(s, w, cfg, temperature) for s in seqs]) if len(seqs) else \
        np.zeros(0, dtype=np.float64)
