"""Oracle: the two trainer-side pieces of the method that consume what the
rollout path emits  (test infrastructure).

1. Decoupled PPO objective (Section 5.2, Eq. 5).  Per token, with the
   behaviour log-prob (emitted at sampling time), the proximal log-prob
   (recomputed over the finished trajectory) and the current policy's log-prob:

       u   = pi_theta / pi_prox
       obj = (pi_prox / pi_behav) * min(u * A, clip(u, 1 - eps, 1 + eps) * A)

   summed over the tokens of the batch.  Forward value only.

2. Dynamic batching (Appendix, Algorithm 1): sequences sorted by length,
   longest first; a sequence opens a new micro-batch while fewer than k_min
   exist or when no existing one has room (total length <= C); otherwise it
   joins, among the micro-batches with room, the one holding the fewest
   sequences.  Reading taken where the text is silent: ties go to the
   micro-batch created first; equal lengths keep their input order; a sequence
   longer than C gets a micro-batch of its own.
"""
from __future__ import annotations

import numpy as np


def decoupled_ppo_objective(logp_theta, logp_prox, logp_behav, adv, eps, mask=None):
    """Returns (sum of the per-token objective, per-token objective, clipped flags)."""
    lt, lp, lb, a = (np.asarray(x, dtype=np.float64) for x in (logp_theta, logp_prox, logp_behav, adv))
    u = np.exp(lt - lp)
    w = np.exp(lp - lb)
    unclipped = u * a
    clipped = np.clip(u, 1.0 - eps, 1.0 + eps) * a
    obj = w * np.minimum(unclipped, clipped)
    is_clipped = clipped < unclipped
    if mask is not None:
        m = np.asarray(mask, dtype=bool)
        obj = np.where(m, obj, 0.0)
        is_clipped = is_clipped & m
    return float(obj.sum()), obj, is_clipped


def dynamic_batching(lengths, capacity, k_min):
    """List of micro-batches, each a list of indices into `lengths`."""
    order = sorted(range(len(lengths)), key=lambda i: -int(lengths[i]))      # stable: ties keep input order
    batches, totals = [], []
    for i in order:
        s = int(lengths[i])
        fits = [b for b in range(len(batches)) if totals[b] + s <= capacity]
        if len(batches) < k_min or not fits:
            batches.append([i])
            totals.append(s)
        else:
            b = min(fits, key=lambda j: (len(batches[j]), j))
            batches[b].append(i)
            totals[b] += s
    return batches
