"""Oracle: the rollout controller's staleness gate  (test infrastructure).

Section 5.1 of the paper: eta is the maximum staleness permitted in a training
batch.  With the current policy version i, the number N_r of trajectories whose
generation has been requested so far and the training batch size B, a new
generation request may be submitted only if, counting it,

    floor((N_r - 1) / B) <= i + eta.

Reading taken: N_r includes the request being submitted (the k-th request,
k = 1, 2, ..., lands in training batch floor((k-1)/B), which is consumed by
training step floor((k-1)/B), i.e. trained on by version floor((k-1)/B); the
inequality bounds that batch index by i + eta).  With eta = 0 this is
synchronous training: a batch is only generated once the previous one has
produced a new version.

The controller below follows the text one request at a time.
"""
from __future__ import annotations


class StalenessGate:
    def __init__(self, batch_size, eta, version=0):
        assert batch_size >= 1 and eta >= 0
        self.B = int(batch_size)
        self.eta = int(eta)
        self.version = int(version)     # i
        self.submitted = 0              # N_r

    def may_submit(self):
        n_r = self.submitted + 1        # counting the request under consideration
        return (n_r - 1) // self.B <= self.version + self.eta

    def submit(self, n):
        """Try to submit n requests one after another; returns how many passed."""
        ok = 0
        for _ in range(int(n)):
            if not self.may_submit():
                break
            self.submitted += 1
            ok += 1
        return ok

    def set_version(self, i):
        assert int(i) >= self.version
        self.version = int(i)


def simulate_stream(n_total, batch_size, eta, slots, lengths):
    """Plain event loop of a streaming rollout with a trainer that steps as soon
    as `batch_size` trajectories have finished: each tick every live trajectory
    emits one token; finished ones free their slot; free slots are refilled
    while the gate admits.  Returns (ticks, list of (request index, version at
    submission, version at completion))."""
    gate = StalenessGate(batch_size, eta)
    live = {}          # request index -> [remaining tokens, version at submission]
    done = []
    finished = 0
    ticks = 0
    nxt = 0
    while len(done) < n_total:
        while len(live) < slots and nxt < n_total and gate.may_submit():
            gate.submit(1)
            live[nxt] = [int(lengths[nxt]), gate.version]
            nxt += 1
        assert live, "the gate closed with nothing in flight: eta too small for this stream to end"
        ticks += 1
        for k in list(live):
            live[k][0] -= 1
            if live[k][0] == 0:
                done.append((k, live[k][1], gate.version))
                del live[k]
                finished += 1
                if finished % batch_size == 0:
                    gate.set_version(gate.version + 1)
    return ticks, done
