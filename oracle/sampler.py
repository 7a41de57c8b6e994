"""Oracle: drawing a_t and reporting log pi_behav(a_t | s_t)  (test infrastructure).

Section 5.2 of the paper needs, for every sampled token, the probability that
the policy *used for sampling* gave it (the denominator of the importance
ratio in the decoupled objective); its Table 3 fixes the generation defaults
temperature 1, top-p 1, top-k off.  The paper does not say how the draw is
made.  Because this build requires the GPU sampler to return the same token
id as this file given the same float32 logits and seed, the draw is specified
here as a procedure whose every step has one possible result:

 1. z_i = logits_i * invT with invT = float32(1)/float32(T); m = max_i z_i.
 2. w_i = sexp(z_i - m): a fixed float32 routine (`sexp` below) in which every
    operation is one individually rounded IEEE float32 multiply, add or
    subtract, so no fused multiply-add and no library exp is involved.
 3. c_i = floor(w_i * 2**32) as an unsigned integer: the fixed-point mass.
    Sums of c_i are integers, so the order of summation cannot matter.
 4. Nucleus: with S = sum c_i and target = clamp(ceil(double(top_p) * S), 1, S),
    rank tokens by (c_i descending, id ascending) and keep the shortest prefix
    of that ranking whose mass reaches target.  top_p >= 1 keeps everything.
 5. Draw: (r0, r1, _, _) = Philox4x32-10(counter = (position, seq_id, 0, 0),
    key = (seed low word, seed high word)); R = r1 * 2**32 + r0;
    r = floor(R * S_nuc / 2**64).  Scan the kept tokens in ascending id order;
    the token is the first whose running mass exceeds r.
 6. log pi_behav = log(c_tok / S_nuc) (the distribution actually drawn from);
    log pi_full = log_softmax(z)[tok] (temperature applied, no truncation).
    A forced token (teacher forcing) skips step 5; if it lies outside the
    nucleus or has c_tok = 0, log pi_behav is -inf.
"""
from __future__ import annotations

import math

import numpy as np

F32 = np.float32
U64 = np.uint64

# ---------------------------------------------------------------- Philox ---
# Philox4x32-10 as published by Salmon, Moraes, Dror and Shaw, "Parallel
# random numbers: as easy as 1, 2, 3" (SC'11): multipliers, Weyl key
# increments, ten rounds.
_PHILOX_M0 = 0xD2511F53
_PHILOX_M1 = 0xCD9E8D57
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """counter: 4 words, key: 2 words (Python ints < 2**32) -> 4 words."""
    c0, c1, c2, c3 = (int(x) & _MASK32 for x in counter)
    k0, k1 = (int(x) & _MASK32 for x in key)
    for rnd in range(10):
        if rnd:
            k0 = (k0 + _PHILOX_W0) & _MASK32
            k1 = (k1 + _PHILOX_W1) & _MASK32
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> 32, p0 & _MASK32
        hi1, lo1 = p1 >> 32, p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & _MASK32, lo1, (hi0 ^ c3 ^ k1) & _MASK32, lo0
    return c0, c1, c2, c3


def draw_u64(seed, seq_id, position):
    """The 64 random bits of step 5 for one (sequence, position)."""
    seed = int(seed)
    r = philox4x32_10((position, seq_id, 0, 0), (seed & _MASK32, (seed >> 32) & _MASK32))
    return (r[1] << 32) | r[0]


# ------------------------------------------------------------------ sexp ---
SEXP_CUTOFF = F32(-25.0)            # below this the mass is zero by definition
_LOG2E = F32(1.4426950408889634)
_LN2_HI = F32(0.693359375)          # 10 significant bits: n * LN2_HI is exact
_LN2_LO = F32(-2.12194440e-4)       # ln 2 - LN2_HI
_TAYLOR = [F32(1.0 / math.factorial(k)) for k in range(8)]   # 1/0! .. 1/7!


def sexp(x):
    """Specified float32 exponential for x <= 0 (array in, array out).

    n = rint(x * log2e) (ties to even); r = (x - n*LN2_HI) - n*LN2_LO;
    p = Horner evaluation of the degree-7 Taylor polynomial of e^r, highest
    coefficient first, each step "p = p * r" then "p = p + coeff";
    result = min(p * 2**n, 1), and 0 where x < -25.  Every operation is a
    single float32 operation rounded to nearest even.
    """
    x = np.asarray(x, dtype=F32)
    xs = np.maximum(x, SEXP_CUTOFF)              # keeps the arithmetic in range
    n = np.rint(xs * _LOG2E).astype(F32)
    r = (xs - n * _LN2_HI).astype(F32)
    r = (r - n * _LN2_LO).astype(F32)
    p = np.full_like(r, _TAYLOR[7])
    for k in range(6, -1, -1):
        p = (p * r).astype(F32)
        p = (p + _TAYLOR[k]).astype(F32)
    w = np.ldexp(p, n.astype(np.int32)).astype(F32)
    w = np.minimum(w, F32(1.0))
    return np.where(x < SEXP_CUTOFF, F32(0.0), w).astype(F32)


def fixed_point_mass(w):
    """c = floor(w * 2**32) as uint64 (exact: power-of-two scale, truncation)."""
    return (np.asarray(w, dtype=np.float64) * 4294967296.0).astype(U64)


def scaled_logits(logits, temperature):
    inv_t = F32(1.0) / F32(temperature)
    return (np.asarray(logits, dtype=F32) * inv_t).astype(F32)


def masses(logits, temperature):
    """Steps 1-3: returns (z, m, c)."""
    z = scaled_logits(logits, temperature)
    m = z.max()
    c = fixed_point_mass(sexp((z - m).astype(F32)))
    return z, m, c


# --------------------------------------------------------------- nucleus ---
def nucleus_target(S, top_p):
    t = math.ceil(float(F32(top_p)) * float(S))
    return min(max(int(t), 1), int(S))


def nucleus(c, top_p):
    """Step 4: boolean membership mask and the integer mass of the kept set."""
    c = np.asarray(c, dtype=U64)
    S = int(c.sum(dtype=U64))
    if F32(top_p) >= F32(1.0):
        return np.ones(c.shape, dtype=bool), S
    target = nucleus_target(S, top_p)
    order = np.argsort(-c.astype(np.int64), kind="stable")   # c desc, id asc
    cum = np.cumsum(c[order], dtype=U64)
    k = int(np.searchsorted(cum, U64(target), side="left"))  # first cum >= target
    keep = np.zeros(c.shape, dtype=bool)
    keep[order[: k + 1]] = True
    return keep, int(cum[k])


# ------------------------------------------------------------------ draw ---
def pick(c, keep, S_nuc, R):
    """Step 5 given the 64 random bits R."""
    r = (int(R) * int(S_nuc)) >> 64
    run = np.cumsum(np.where(keep, c, U64(0)), dtype=U64)
    return int(np.searchsorted(run, U64(r), side="right"))   # first run > r


def sample_row(logits, temperature, top_p, seed, seq_id, position, forced=None):
    """All six steps for one row.  Returns (token, logp_behav, logp_full)."""
    z, m, c = masses(logits, temperature)
    keep, S_nuc = nucleus(c, top_p)
    if forced is None:
        tok = pick(c, keep, S_nuc, draw_u64(seed, seq_id, position))
    else:
        tok = int(forced)
    ct = int(c[tok])
    if keep[tok] and ct > 0:
        logp_behav = math.log(ct) - math.log(S_nuc)
    else:
        logp_behav = -math.inf
    zd = z.astype(np.float64) - float(m)
    logp_full = float(zd[tok]) - math.log(float(np.sum(np.exp(zd))))
    return tok, logp_behav, logp_full


def sample_batch(logits, temperature, top_p, seed, seq_ids, positions, forced=None):
    """Row-by-row `sample_row` over logits [n, V]."""
    n = len(seq_ids)
    toks = np.empty(n, dtype=np.int32)
    lb = np.empty(n, dtype=np.float64)
    lf = np.empty(n, dtype=np.float64)
    for i in range(n):
        f = None if forced is None else int(forced[i])
        toks[i], lb[i], lf[i] = sample_row(logits[i], temperature, top_p, seed,
                                           int(seq_ids[i]), int(positions[i]), f)
    return toks, lb, lf
