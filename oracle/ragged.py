"""Ragged batches on the CPU oracle (test infrastructure only, never imported by the product).

Alg. 1 keeps one budgeted cache per sequence: the counters t (tokens seen) and n (resident rows),
the threshold 1/t of Alg. 2, the history window and the moments at which a compression is due
all belong to that sequence.  A batch whose sequences have different prompt lengths, or stop
generating at different steps, is therefore nothing but independent runs of Alg. 1, one per
sequence; this module writes exactly that: one single-sequence `Oracle` per batch entry, stepped
only when the sequence takes part in a step and compressed only when its own cache is due.
"""
from __future__ import annotations

import dataclasses

import numpy as np

from oracle.sco import Oracle, OracleConfig


class RaggedOracle:
    """`cfg.batch` sequences of `cfg.heads` units each, every sequence with its own t and n."""

    def __init__(self, cfg: OracleConfig, nthreads: int | None = None):
        self.cfg = cfg
        self.batch, self.heads, self.d = cfg.batch, cfg.heads, cfg.head_dim
        self.U = cfg.batch * cfg.heads
        one = dataclasses.replace(cfg, batch=1)
        self.seq = [Oracle(one, nthreads) for _ in range(cfg.batch)]
        self.cap = self.seq[0].cap

    def lengths(self):
        """(n [batch], t [batch])."""
        ln = [s.lengths() for s in self.seq]
        return np.array([x[0] for x in ln], dtype=np.int64), np.array([x[1] for x in ln], dtype=np.int64)

    def _units(self, b):
        return slice(b * self.heads, (b + 1) * self.heads)

    def step(self, q, k_new, v_new, active=None, p_forced=None):
        """One step of every sequence with active[b] true (all when None).  q, k_new, v_new are
        [U, d]; rows of idle sequences are ignored.  Returns (out [U, d] f64, probs [U, cap] f64,
        due [batch] bool); rows of idle sequences are NaN, their `due` false."""
        act = np.ones(self.batch, dtype=bool) if active is None else np.asarray(active, dtype=bool)
        q, k_new, v_new = (np.asarray(a).reshape(self.U, self.d) for a in (q, k_new, v_new))
        out = np.full((self.U, self.d), np.nan)
        probs = np.full((self.U, self.cap), np.nan)
        due = np.zeros(self.batch, dtype=bool)
        for b in range(self.batch):
            if not act[b]:
                continue
            u = self._units(b)
            pf = None if p_forced is None else p_forced[u]
            out[u], probs[u], due[b] = self.seq[b].step(q[u], k_new[u], v_new[u], p_forced=pf)
        return out, probs, due

    def due(self):
        """Sequences whose cache stands at its trigger size (a compression is due)."""
        n, _ = self.lengths()
        return n == self.cap_rows()

    def cap_rows(self):
        c = self.cfg
        return c.budget + (c.drop if c.trigger == 1 else 1)

    def compress(self):
        """Alg. 2 on every sequence that is due.  Returns evicted [U, m] int32, rows of the
        sequences that were not due filled with -1."""
        ev = np.full((self.U, self.cfg.drop), -1, dtype=np.int32)
        for b in np.flatnonzero(self.due()):
            ev[self._units(b)] = self.seq[b].compress()
        return ev

    def importance(self, b):
        return self.seq[b].importance()

    def positions(self, b):
        return self.seq[b].positions()

    def rows(self, b):
        return self.seq[b].rows()
