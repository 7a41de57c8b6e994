"""CPU oracle for the rollout worker's generation path (test infrastructure).

This package is the slow, plain reference that the HIP library is checked
against.  It is test infrastructure only: nothing in the product package may
import it, and it imports nothing from the product package.  Everything here
is numpy on the host, float64 for the decoder arithmetic and exact integer /
individually rounded float32 operations for the sampler.

Modules
-------
decoder  -- the decoder-only policy pi_theta(a_t | q, a_<t) of Section 3.1:
            one dense causal forward pass per prefix (the plain definition),
            plus an incremental-KV variant used to prove the cache invariant.
sampler  -- the specified sampling procedure that draws a_t and reports
            log pi_behav(a_t | s_t) for the decoupled objective (Section 5.2).
rollout  -- generate / update_weights semantics of the interruptible rollout
            worker (Section 4.1) and the per-position policy versions of
            Proposition 1.
scoring  -- teacher-forced log-probabilities of whole trajectories: the
            proximal policy's token probabilities that the decoupled objective
            recomputes when a training batch arrives (Section 5.2, Eq. 5).
staleness -- the staleness gate floor((N_r - 1) / B) <= i + eta of the rollout
            controller and a plain event loop of the streaming regime
            (Sections 4.1, 5.1).
trainer_side -- the decoupled PPO objective (Section 5.2, Eq. 5, forward value)
            and the dynamic batching procedure (Algorithm 1).

Pins (tests that tie each function to something other than itself) live in
tests/test_oracle_*.py.  Parity status per function:

decoder.rmsnorm, rope, attention, swiglu, forward  -- pinned (closed forms,
    brute force, invariances).
decoder whole-model values -- pinned: the full forward pass agrees with the public
    Qwen2 model class of the `transformers` library in float64 on random weights
    (test_forward_matches_public_qwen2_implementation); no trained checkpoint is
    involved anywhere in this build.
sampler.philox4x32_10 -- pinned by the known-answer vectors distributed with
    the generator's reference implementation (tests/golden/philox_kat.txt).
sampler.sexp, mass, nucleus, draw, logprobs -- pinned (libm, exact integer
    identities, brute-force sort, chi-square on empirical frequencies).
scoring.sequence_logprobs -- pinned (log-softmax closed forms, agreement with
    the rollout oracle's emitted log-probs, tests/test_oracle_scoring.py).
staleness.StalenessGate, simulate_stream -- pinned (the synchronous schedule
    at eta = 0, brute-force enumeration, tests/test_oracle_staleness.py).
trainer_side.decoupled_ppo_objective, dynamic_batching -- pinned (reduction to the
    standard clipped objective when prox = behav, brute force on small inputs,
    tests/test_oracle_trainer_side.py).
"""
