"""Pins for oracle/sampler.py."""
import math
import os

import numpy as np
import pytest

from oracle import sampler

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------- philox
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        assert list(sampler.philox4x32_10(w[0:4], w[4:6])) == w[6:10]


def test_draw_u64_word_order_and_counter_layout():
    # R = r1 * 2**32 + r0 of Philox(counter=(position, seq_id, 0, 0), key=(lo, hi))
    seed = (0x299F31D0 << 32) | 0xA4093822
    r = sampler.philox4x32_10((7, 3, 0, 0), (0xA4093822, 0x299F31D0))
    assert sampler.draw_u64(seed, seq_id=3, position=7) == (r[1] << 32) | r[0]
    assert sampler.draw_u64(seed, 3, 7) != sampler.draw_u64(seed, 7, 3)


def test_philox_uniformity():
    # 64 buckets over 20000 draws: chi-square far below a gross-failure bound
    counts = np.zeros(64)
    for p in range(20000):
        counts[sampler.draw_u64(123, 5, p) >> 58] += 1
    chi2 = ((counts - 312.5) ** 2 / 312.5).sum()
    assert chi2 < 120.0           # 63 dof: P(chi2 > 120) ~ 1e-5


# --------------------------------------------------------------------- sexp
def test_sexp_close_to_libm_exp():
    x = np.linspace(-25.0, 0.0, 400001).astype(np.float32)
    ref = np.exp(x.astype(np.float64))
    rel = np.abs(sampler.sexp(x).astype(np.float64) - ref) / ref
    assert rel.max() < 4 * 2.0 ** -24


def test_sexp_special_values():
    assert sampler.sexp(np.float32(0.0)) == np.float32(1.0)
    assert sampler.sexp(np.float32(-25.5)) == 0.0
    assert sampler.sexp(np.float32(-1e30)) == 0.0
    w = sampler.sexp(-np.abs(np.random.default_rng(0).standard_normal(10000)).astype(np.float32))
    assert w.dtype == np.float32 and (w <= 1).all() and (w > 0).all()


def test_sexp_every_step_is_a_float32_operation():
    # the same steps with Python floats rounded to float32 after each operation
    f = lambda v: float(np.float32(v))
    for x in [-0.1, -0.3465, -0.3467, -1.0, -7.77, -22.18, -24.99]:
        x = f(x)
        n = float(np.rint(np.float32(f(x * f(1.4426950408889634)))))
        r = f(f(x - f(n * 0.693359375)) - f(n * f(-2.12194440e-4)))
        p = f(1.0 / 5040.0)
        for k in (720.0, 120.0, 24.0, 6.0, 2.0, 1.0, 1.0):
            p = f(f(p * r) + f(1.0 / k))
        want = min(f(p * 2.0 ** n), 1.0)
        assert float(sampler.sexp(np.float32(x))) == want


def test_fixed_point_mass_exact():
    w = np.array([1.0, 0.5, 2.0 ** -32, 2.0 ** -33, 0.75 + 2.0 ** -24, 0.0], dtype=np.float32)
    c = sampler.fixed_point_mass(w)
    assert c.tolist() == [2 ** 32, 2 ** 31, 1, 0, 3 * 2 ** 30 + 2 ** 8, 0]


# ------------------------------------------------------------------ nucleus
def _brute_nucleus(c, top_p):
    S = sum(c)
    if np.float32(top_p) >= 1:
        return set(range(len(c))), S
    target = min(max(math.ceil(float(np.float32(top_p)) * S), 1), S)
    ranked = sorted(range(len(c)), key=lambda i: (-c[i], i))
    tot, keep = 0, set()
    for i in ranked:
        keep.add(i)
        tot += c[i]
        if tot >= target:
            break
    return keep, tot


@pytest.mark.parametrize("top_p", [1.0, 0.95, 0.5, 0.1, 1e-6])
def test_nucleus_matches_brute_force_with_ties(top_p):
    rng = np.random.default_rng(int(top_p * 1000))
    for trial in range(30):
        c = rng.integers(0, 6, size=40).astype(np.uint64) * np.uint64(1000)   # many ties, zeros
        c[rng.integers(0, 40)] = 2 ** 32
        keep, S_nuc = sampler.nucleus(c, top_p)
        bk, bs = _brute_nucleus([int(x) for x in c], top_p)
        assert set(np.nonzero(keep)[0].tolist()) == bk and S_nuc == bs


def test_nucleus_selection_form_equivalence():
    # the kept set = all masses above a threshold tau plus the lowest-id
    # ceil((target - mass_above) / tau) tokens with mass exactly tau
    rng = np.random.default_rng(5)
    for trial in range(50):
        c = rng.integers(1, 9, size=64).astype(np.uint64)
        top_p = float(rng.uniform(0.05, 0.99))
        keep, S_nuc = sampler.nucleus(c, top_p)
        S = int(c.sum())
        target = sampler.nucleus_target(S, top_p)
        tau = int(c[keep].min())
        above = int(c[c > tau].sum())
        assert above < target <= int(c[c >= tau].sum())
        n_tie = -(-(target - above) // tau)
        want = (c > tau)
        want[np.nonzero(c == tau)[0][:n_tie]] = True
        assert (want == keep).all() and S_nuc == above + n_tie * tau


def test_nucleus_limits():
    c = np.array([5, 9, 9, 1], dtype=np.uint64)
    keep, S = sampler.nucleus(c, 1.0)
    assert keep.all() and S == 24
    keep, S = sampler.nucleus(c, 1e-9)       # -> argmax, lowest id on ties
    assert keep.tolist() == [False, True, False, False] and S == 9
    # minimality: dropping the last-ranked member falls below the target
    keep, S = sampler.nucleus(c, 0.8)        # target = ceil(0.8*24 (float32 0.8)) = 20
    assert keep.tolist() == [True, True, True, False] and S == 23 and S - 5 < 20


# --------------------------------------------------------------------- draw
def test_pick_is_inverse_cdf_in_id_order():
    c = np.array([3, 0, 5, 2], dtype=np.uint64)
    keep = np.array([True, True, True, False])
    S = 8
    toks = [sampler.pick(c, keep, S, (r << 64) // S + (1 if (r << 64) % S else 0))
            for r in range(S)]           # smallest R with floor(R*S/2^64) = r
    assert toks == [0, 0, 0, 2, 2, 2, 2, 2]
    assert sampler.pick(c, keep, S, 2 ** 64 - 1) == 2


def test_empirical_frequencies_match_masses():
    rng = np.random.default_rng(7)
    logits = (rng.standard_normal(12) * 1.5).astype(np.float32)
    for temperature, top_p in [(1.0, 1.0), (0.7, 0.9)]:
        z, m, c = sampler.masses(logits, temperature)
        keep, S_nuc = sampler.nucleus(c, top_p)
        probs = np.where(keep, c, 0).astype(np.float64) / S_nuc
        n = 40000
        counts = np.zeros(12)
        for p in range(n):
            tok, lb, lf = sampler.sample_row(logits, temperature, top_p, 99, 4, p)
            counts[tok] += 1
            assert keep[tok]
        sel = probs > 0
        chi2 = ((counts[sel] - n * probs[sel]) ** 2 / (n * probs[sel])).sum()
        assert counts[~sel].sum() == 0
        assert chi2 < 45.0        # <= 11 dof: P(chi2 > 45) < 1e-5


# ---------------------------------------------------------------- log-probs
def test_logprobs_at_defaults_equal_log_softmax():
    rng = np.random.default_rng(8)
    logits = rng.standard_normal(1000).astype(np.float32)
    ls = logits.astype(np.float64)
    ls = ls - ls.max()
    ls = ls - math.log(np.exp(ls).sum())
    for pos in range(5):
        tok, lb, lf = sampler.sample_row(logits, 1.0, 1.0, 1, 0, pos)
        assert abs(lf - ls[tok]) < 1e-12
        assert abs(lb - ls[tok]) < 1e-5       # 2**-32 quantisation + sexp error
    z, m, c = sampler.masses(logits, 1.0)
    assert abs(np.exp(np.log(c.astype(np.float64)) - math.log(int(c.sum()))).sum() - 1) < 1e-9


def test_temperature_and_truncation_in_logprobs():
    logits = np.array([2.0, 1.0, 0.0, -1.0], dtype=np.float32)
    tok, lb, lf = sampler.sample_row(logits, 0.5, 1.0, 0, 0, 0, forced=1)
    z = np.array([4.0, 2.0, 0.0, -2.0])
    assert abs(lf - (2.0 - math.log(np.exp(z).sum()))) < 1e-12
    # top-p small: only token 0 is kept; forcing token 1 reports -inf behaviour log-prob
    tok, lb, lf = sampler.sample_row(logits, 1.0, 0.3, 0, 0, 0, forced=1)
    assert tok == 1 and lb == -math.inf and math.isfinite(lf)
    tok, lb, lf = sampler.sample_row(logits, 1.0, 0.3, 0, 0, 0, forced=0)
    assert lb == 0.0
    # renormalisation over the kept set {0, 1} at top_p = 0.8
    tok, lb, lf = sampler.sample_row(logits, 1.0, 0.8, 0, 0, 0, forced=1)
    assert abs(lb - math.log(math.e / (math.e ** 2 + math.e))) < 1e-6


def test_forced_token_with_zero_mass():
    logits = np.array([0.0, -30.0, -1.0], dtype=np.float32)
    tok, lb, lf = sampler.sample_row(logits, 1.0, 1.0, 0, 0, 0, forced=1)
    assert lb == -math.inf and abs(lf - (-30.0 - math.log(1 + math.exp(-30) + math.exp(-1)))) < 1e-9
