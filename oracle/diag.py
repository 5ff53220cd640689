"""Plain reference of the diagnostics the paper plots (TEST INFRASTRUCTURE ONLY, like the rest
of ``oracle/``; the product never imports it).

* Persistence ratio, Sec. 3.1 ("Verification"): a token is pivotal for position t when it gets
  more than 1/t of that position's attention; S(0->t) and S(t+1->l) are the unions of the
  pivotal sets over the first t and the later positions, both over the tokens x_1..x_t; the ratio
  is |S(t+1->l) & S(0->t)| / |S(t+1->l)|.
* Attention-score change ratio, Sec. 5 (ablation on the attention score error):
  (a_s - a_o)/a_o per token, a_o the full-attention score, a_s the budgeted one (0 if evicted).
  By the restricted-softmax identity in the proof of Lemma A.4, a_s = a_o / mass for every
  survivor, mass = full attention held by the survivors.
"""
from __future__ import annotations

import numpy as np


def pivotal_sets(probs, split):
    """probs[i][j], j <= i: attention of position i (0-based, t = i+1 tokens seen) on token j.
    Returns (S_first, S_later) as sets of tokens j < split; the comparison is made in fp32 on
    the fp32 value of the probability against 1.0f/(float)t, strict."""
    first, later = set(), set()
    T = len(probs)
    for i in range(T):
        tau = np.float32(1.0) / np.float32(i + 1)
        for j in range(min(i + 1, split)):
            if np.float32(probs[i][j]) > tau:
                (first if i < split else later).add(j)
    return first, later


def persistence_counts(probs, split):
    """-> (|S_first|, |S_later|, |S_first & S_later|); ratio = third / second."""
    first, later = pivotal_sets(probs, split)
    return len(first), len(later), len(first & later)


def kept_mass(positions, probs_full):
    """Full-attention mass on the resident tokens: sum of probs_full[p] over their positions."""
    return float(sum(float(probs_full[int(p)]) for p in positions))


def change_ratio(a_s, a_o):
    return (np.asarray(a_s, dtype=np.float64) - np.asarray(a_o, dtype=np.float64)) / np.asarray(a_o, dtype=np.float64)
