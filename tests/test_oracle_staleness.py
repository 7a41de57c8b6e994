"""Pins for oracle/staleness.py (Section 5.1 staleness gate): the synchronous
special case eta = 0, the closed form of the admitted count, the staleness of
every training batch in a simulated stream, and monotonicity in eta."""
import numpy as np

from oracle import staleness


def test_eta_zero_is_synchronous():
    """eta = 0: exactly one batch may be requested per policy version."""
    g = staleness.StalenessGate(batch_size=4, eta=0)
    assert g.submit(10) == 4 and g.submit(1) == 0
    g.set_version(1)
    assert g.submit(10) == 4 and g.submitted == 8
    g.set_version(3)                                   # two versions at once: two more batches
    assert g.submit(100) == 8 and g.submitted == 16


def test_admitted_count_closed_form():
    """floor((N-1)/B) <= i + eta  <=>  N <= (i + eta + 1) B: checked for every
    small (B, eta, i) by submitting without limit."""
    for B in range(1, 7):
        for eta in range(0, 4):
            g = staleness.StalenessGate(B, eta)
            for i in range(0, 5):
                g.set_version(i)
                g.submit(10 ** 4)
                assert g.submitted == (i + eta + 1) * B
                assert not g.may_submit()


def test_stream_keeps_every_batch_within_eta():
    """In a simulated stream the trajectories of training batch b (requests
    bB .. bB+B-1) were all submitted under a version >= b - eta."""
    rng = np.random.default_rng(0)
    for eta in (0, 1, 3):
        B, n = 8, 96
        lengths = rng.integers(1, 60, size=n)
        ticks, done = staleness.simulate_stream(n, B, eta, slots=16, lengths=lengths)
        assert len(done) == n
        for k, v_sub, v_done in done:
            assert k // B - v_sub <= eta
            assert v_done >= v_sub


def test_larger_eta_never_slows_the_stream():
    rng = np.random.default_rng(1)
    lengths = np.clip(np.round(np.exp(rng.normal(3.0, 1.0, size=128))), 1, 200).astype(int)
    t = [staleness.simulate_stream(128, 16, eta, slots=32, lengths=lengths)[0] for eta in (0, 1, 2, 4, 8)]
    assert all(a >= b for a, b in zip(t, t[1:])) and t[0] > t[-1]
