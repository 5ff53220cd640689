"""Pins of the ragged-batch oracle (CPU only): Alg. 1 applied to each sequence on its own."""
import numpy as np
import pytest

from oracle import sco
from oracle.ragged import RaggedOracle
from oracle.sco import Oracle, OracleConfig


def _inputs(rng, U, T, d):
    return tuple(rng.standard_normal((U, T, d)).astype(np.float16) for _ in range(3))


@pytest.mark.parametrize("trigger", [sco.HARD_CAP, sco.HIGH_WATER])
def test_equal_lengths_reduce_to_the_lock_step_batch(trigger):
    """With every sequence active at every step the ragged oracle is the batched oracle, bit for
    bit: outputs, probabilities, due steps, evicted slots, positions and stored rows."""
    cfg = OracleConfig(3, 2, 64, sco.F16, 20, 3, 8, 4, trigger)
    rng = np.random.default_rng(1)
    U, T = 6, 60
    q, k, v = _inputs(rng, U, T, 64)
    a, b = RaggedOracle(cfg), Oracle(cfg)
    for s in range(T):
        oa, pa, due_a = a.step(q[:, s], k[:, s], v[:, s])
        ob, pb, due_b = b.step(q[:, s], k[:, s], v[:, s])
        n = b.n
        assert np.array_equal(oa, ob) and np.array_equal(pa[:, :n], pb[:, :n])
        assert np.all(due_a == due_b)
        if due_b:
            assert np.array_equal(a.compress(), b.compress())
    for s_ in range(3):
        u = slice(2 * s_, 2 * s_ + 2)
        assert np.array_equal(a.positions(s_), b.positions()[u])
        assert np.array_equal(a.rows(s_)[0], b.rows()[0][u])


def test_each_sequence_follows_its_own_clock():
    """Sequences that started with prompts of different lengths become due at their own steps
    t_b = n_trig + k*m, use their own threshold 1/t_b, and are unaffected by the steps they sit
    out: a sequence stepped only every other step ends exactly like the same sequence stepped
    alone with the same inputs."""
    cfg = OracleConfig(3, 2, 64, sco.F16, 12, 2, 6, 3)
    n_trig = 13
    rng = np.random.default_rng(2)
    T = 70
    q, k, v = _inputs(rng, 6, T, 64)
    rag = RaggedOracle(cfg)
    solo = [Oracle(OracleConfig(1, 2, 64, sco.F16, 12, 2, 6, 3)) for _ in range(3)]
    taken = [0, 0, 0]   # inputs consumed by each sequence
    due_at = [[], [], []]
    for s in range(T):
        active = np.array([True, s % 2 == 0, s >= 25])
        idle_before = [rag.seq[b].lengths() for b in range(3)]
        out, probs, due = rag.step(q[:, s], k[:, s], v[:, s], active)
        for b in range(3):
            u = slice(2 * b, 2 * b + 2)
            if not active[b]:
                assert rag.seq[b].lengths() == idle_before[b] and not due[b]
                assert np.all(np.isnan(out[u]))
                continue
            o, p, d_ = solo[b].step(q[u, s], k[u, s], v[u, s])
            taken[b] += 1
            assert np.array_equal(out[u], o) and d_ == due[b]
            if d_:
                due_at[b].append(solo[b].t)
        ev = rag.compress()
        for b in range(3):
            u = slice(2 * b, 2 * b + 2)
            if due[b]:
                assert np.array_equal(ev[u], solo[b].compress())
            else:
                assert np.all(ev[u] == -1)
    n, t = rag.lengths()
    assert list(t) == taken == [70, 35, 45]
    for b in range(3):
        assert due_at[b] == list(range(n_trig, taken[b] + 1, 3))
        assert np.array_equal(rag.positions(b), solo[b].positions())


def test_threshold_uses_the_sequence_own_token_count():
    """The low-score threshold of a sequence is 1/t_b of that sequence.  With equal keys every
    probability is 1/n >= 1/t, never low; a forced probability of 0.15 is low for a sequence at
    t <= 6 (1/6 > 0.15) and not low for one at t >= 7 (1/7 < 0.15), at the very same call."""
    cfg = OracleConfig(2, 1, 64, sco.F16, 6, 1, 4, 2)
    rag = RaggedOracle(cfg)
    k1 = np.ones((2, 64), dtype=np.float16)
    # sequence 0 takes 9 steps (compressed at t = 7 and 9), sequence 1 only the last 5
    for s in range(9):
        active = np.array([True, s >= 4])
        _, _, due = rag.step(k1, k1, k1, active)
        rag.compress()
    n, t = rag.lengths()
    assert list(t) == [9, 5] and list(n) == [5, 5]
    # sequence 1: n == t at every step, p = 1/n = 1/t is not below the threshold: empty record
    assert np.all(rag.importance(1) == 0)
    # sequence 0: since its first compression n < t, so p = 1/n > 1/t: never low either; the
    # record differs only through t when probabilities fall between 1/t_0 and 1/t_1
    assert np.all(rag.importance(0) == 0)
    # a probability of 0.15 is low for t = 5 (1/5) but not for t = 9 (1/9): force it
    pf = np.full((2, 8), 0.15, dtype=np.float32)
    rag2 = RaggedOracle(cfg)
    for s in range(9):
        active = np.array([True, s >= 4])
        rag2.step(k1, k1, k1, active, p_forced=pf)
        if s < 8:
            rag2.compress()
    # sequence 1 (t = 1..5): 0.15 < 1/t for every step; sequence 0 at t = 7, 8, 9: 0.15 > 1/t
    assert rag2.importance(1).min() >= 1
    I0 = rag2.importance(0)
    assert I0[0, -1] == 0 and I0[0, -2] == 0  # rows appended at t = 8, 9 were never low
