"""Oracle: the interruptible rollout worker  (test infrastructure).

Section 4.1 of the paper gives the worker two requests.  `generate` produces
responses for prompts; `update_weights` interrupts every generation in flight,
loads the new parameters, throws away the KV cache computed with the old ones,
recomputes it with the new ones and goes on decoding.  A trajectory therefore
consists of segments produced by different policy versions, and Proposition 1
(Section 5.2, Appendix D) says its behaviour policy is defined position by
position: the token at position t was drawn from whichever version was loaded
when it was sampled, and that never changes afterwards.

In the plain definition used here there is no cache at all: the logits for the
next token are always `decoder.next_logits` of the whole prefix under the
weights loaded now.  `update_weights` is then nothing but a switch of the
weight set.  With `use_cache=True` the worker keeps K and V per sequence and
really discards and rebuilds them on update; that variant exists to show that
both behave the same.
"""
from __future__ import annotations

import numpy as np

from . import decoder, sampler


class RolloutWorker:
    def __init__(self, cfg, weights, version, seed, temperature=1.0, top_p=1.0,
                 use_cache=False):
        self.cfg = cfg
        self.w = weights
        self.version = int(version)
        self.seed = int(seed)
        self.temperature = temperature
        self.top_p = top_p
        self.use_cache = use_cache
        self.tokens = {}        # seq_id -> list of token ids (prompt + generated)
        self.prompt_len = {}
        self.logp_behav = {}    # seq_id -> list, one per generated token
        self.logp_full = {}
        self.versions = {}      # seq_id -> list, policy version per generated token
        self.finished = set()
        self._dec = {}          # seq_id -> IncrementalDecoder (use_cache only)
        self._logits = {}       # seq_id -> cached next-token logits (use_cache only)

    # -- generate ---------------------------------------------------------
    def add(self, seq_id, prompt):
        self.tokens[seq_id] = [int(t) for t in prompt]
        self.prompt_len[seq_id] = len(prompt)
        self.logp_behav[seq_id] = []
        self.logp_full[seq_id] = []
        self.versions[seq_id] = []
        if self.use_cache:
            self._dec[seq_id] = decoder.IncrementalDecoder(self.w, self.cfg)
            self._logits[seq_id] = self._dec[seq_id].append(self.tokens[seq_id])

    def next_logits(self, seq_id):
        """float64 logits for the token at position len(tokens[seq_id])."""
        if self.use_cache:
            return self._logits[seq_id]
        return decoder.next_logits(self.tokens[seq_id], self.w, self.cfg)

    def step(self, seq_ids, forced=None):
        """Sample (or force) one token for each listed live sequence and append
        it.  Returns (float32 logits [n,V] the tokens were drawn from, tokens)."""
        out_logits, out_tok = [], []
        for i, s in enumerate(seq_ids):
            assert s not in self.finished
            lg = self.next_logits(s).astype(np.float32)
            pos = len(self.tokens[s])
            f = None if forced is None else int(forced[i])
            tok, lb, lf = sampler.sample_row(lg, self.temperature, self.top_p,
                                             self.seed, s, pos, f)
            self.tokens[s].append(tok)
            self.logp_behav[s].append(lb)
            self.logp_full[s].append(lf)
            self.versions[s].append(self.version)
            if self.use_cache:
                self._logits[s] = self._dec[s].append([tok])
            out_logits.append(lg)
            out_tok.append(tok)
        return np.stack(out_logits), np.asarray(out_tok, dtype=np.int32)

    def finish(self, seq_id):
        self.finished.add(seq_id)
        self._dec.pop(seq_id, None)
        self._logits.pop(seq_id, None)

    def live(self):
        return [s for s in self.tokens if s not in self.finished]

    # -- update_weights -----------------------------------------------------
    def update_weights(self, new_weights, new_version):
        """Interrupt: load the new parameters; every unfinished sequence goes on
        from its full prefix under them.  Emitted tokens, their log-probs and
        their version tags are left as they are."""
        assert int(new_version) >= self.version
        self.w = new_weights
        self.version = int(new_version)
        if self.use_cache:
            for s in self.live():
                d = decoder.IncrementalDecoder(self.w, self.cfg)   # old K,V dropped
                self._dec[s] = d
                self._logits[s] = d.append(self.tokens[s])         # recomputed
