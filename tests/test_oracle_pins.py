"""Pins of the CPU oracle against what the paper and the mathematics fix (CPU only).

Each test states the passage it rests on.  None of them re-types the oracle's own
formulas: they use a library softmax, brute-force enumeration, closed forms, an
independently formulated counter, or invariants.
"""
import itertools

import numpy as np
import pytest
import torch

from oracle import sco
from oracle.sco import Oracle, OracleConfig


def _cfg(**kw):
    base = dict(batch=1, heads=2, head_dim=16, kv_dtype=sco.F32, budget=8, recent=2,
                history=4, drop=2)
    base.update(kw)
    return OracleConfig(**base)


def _rand(rng, U, T, d, dtype=np.float32):
    return tuple(rng.standard_normal((U, T, d)).astype(dtype) for _ in range(3))


def _run(o, q, k, v, on_compress=None, p_forced=None):
    """Drive Alg. 1: step, compress when due.  Returns per-step (out, probs, n_at_step)."""
    rec = []
    for s in range(q.shape[1]):
        out, probs, due = o.step(q[:, s], k[:, s], v[:, s])
        rec.append((out, probs, o.n))
        if due:
            I = o.importance()
            pos = o.positions()
            ev = o.compress()
            if on_compress:
                on_compress(s, I, pos, ev)
    return rec


# --------------------------------------------------------------------------------------
# Sec. 4.2, remark after Thm 4.1: with B = T_max nothing is dropped and the error is zero,
# i.e. the path is plain softmax attention (Sec. 4.1, first display).
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,kv", [(np.float32, sco.F32), (np.float16, sco.F16)])
def test_budget_at_least_length_is_textbook_attention(dtype, kv):
    rng = np.random.default_rng(1)
    U, T, d = 3, 40, 16
    q, k, v = _rand(rng, U, T, d, dtype)
    o = Oracle(_cfg(heads=U, head_dim=d, kv_dtype=kv, budget=T, recent=4, history=8, drop=4))
    for s in range(T):
        out, probs, due = o.step(q[:, s], k[:, s], v[:, s])
        if s < T - 1:
            assert not due
        qs = torch.from_numpy(q[:, s].astype(np.float64))
        Ks = torch.from_numpy(k[:, : s + 1].astype(np.float64))
        Vs = torch.from_numpy(v[:, : s + 1].astype(np.float64))
        logits = torch.einsum("ud,usd->us", qs, Ks) / np.sqrt(d)
        p_ref = torch.softmax(logits, dim=-1)
        o_ref = torch.einsum("us,usd->ud", p_ref, Vs)
        np.testing.assert_allclose(probs[:, : s + 1], p_ref.numpy(), rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(out, o_ref.numpy(), rtol=1e-11, atol=1e-13)
        assert np.all(probs[:, s + 1:] == 0.0)


def test_explicit_scale_is_used():
    rng = np.random.default_rng(2)
    q, k, v = _rand(rng, 1, 6, 8)
    o = Oracle(_cfg(heads=1, head_dim=8, budget=16, scale=0.37))
    for s in range(6):
        out, probs, _ = o.step(q[:, s], k[:, s], v[:, s])
    lg = 0.37 * (k[0].astype(np.float64) @ q[0, 5].astype(np.float64))
    p = np.exp(lg - lg.max())
    p /= p.sum()
    np.testing.assert_allclose(probs[0, :6], p, rtol=1e-12)
    np.testing.assert_allclose(out[0], p @ v[0].astype(np.float64), rtol=1e-11, atol=1e-13)


# Sec. 4.1: the estimator's weights are a softmax over the resident rows.
def test_probabilities_sum_to_one_under_compression():
    rng = np.random.default_rng(3)
    q, k, v = _rand(rng, 4, 90, 16)
    o = Oracle(_cfg(heads=4, budget=16, recent=3, history=8, drop=4))
    for out, probs, n in _run(o, q, k, v):
        assert np.all(probs >= 0)
        np.testing.assert_allclose(probs.sum(axis=1), 1.0, rtol=0, atol=1e-12)


# --------------------------------------------------------------------------------------
# Alg. 1 ("if n > B compress such that n <= B"), Alg. 2 ("n <- n - m"), Sec. 4.2
# ("when m = 1 ... the cache will always maintain B tokens").
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("trigger", [sco.HARD_CAP, sco.HIGH_WATER])
@pytest.mark.parametrize("B,r,w,m", [(16, 3, 8, 4), (10, 1, 5, 1), (12, 4, 6, 6), (9, 8, 4, 2)])
def test_cache_size_invariants(trigger, B, r, w, m):
    rng = np.random.default_rng(4)
    T = 70
    q, k, v = _rand(rng, 2, T, 8)
    o = Oracle(_cfg(heads=2, head_dim=8, budget=B, recent=r, history=w, drop=m, trigger=trigger))
    n_trig = B + 1 if trigger == sco.HARD_CAP else B + m
    n_prev = 0
    compress_steps = []
    for s in range(T):
        _, _, due = o.step(q[:, s], k[:, s], v[:, s])
        assert o.n == n_prev + 1 and o.t == s + 1
        assert due == (o.n == n_trig)
        if due:
            o.compress()
            compress_steps.append(s + 1)
            assert o.n == n_trig - m
            if trigger == sco.HARD_CAP:
                assert o.n <= B
                if m == 1:
                    assert o.n == B
            else:
                assert o.n == B
        n_prev = o.n
        assert o.n <= n_trig
    # compressions come every m tokens once the trigger size has been reached
    assert compress_steps[0] == n_trig
    assert all(b - a == m for a, b in zip(compress_steps, compress_steps[1:]))


def test_step_refused_while_due_and_compress_refused_when_not_due():
    rng = np.random.default_rng(5)
    q, k, v = _rand(rng, 1, 12, 8)
    o = Oracle(_cfg(heads=1, head_dim=8, budget=4, recent=1, history=2, drop=2))
    with pytest.raises(RuntimeError):
        o.compress()
    for s in range(5):
        _, _, due = o.step(q[:, s], k[:, s], v[:, s])
    assert due
    with pytest.raises(RuntimeError):
        o.step(q[:, 5], k[:, 5], v[:, 5])
    o.compress()
    o.step(q[:, 5], k[:, 5], v[:, 5])


def test_bad_configs_rejected():
    with pytest.raises(ValueError):
        Oracle(_cfg(budget=4, recent=4, drop=2))  # m > n_trig - r
    with pytest.raises(ValueError):
        Oracle(_cfg(kv_dtype=sco.I4G64, head_dim=32))
    with pytest.raises(ValueError):
        Oracle(_cfg(drop=0))


# --------------------------------------------------------------------------------------
# Sec. 4.1 "recent tokens are always kept"; Alg. 2 keep-set = all but the m largest records.
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(6))
def test_selection_recent_window_optimality_and_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    B, r, w, m = 11, 3, 5, 3
    U, T, d = 3, 60, 8
    q, k, v = _rand(rng, U, T, d)
    # low-entropy logits so that records have many distinct values and many ties
    q *= 3.0
    o = Oracle(_cfg(heads=U, head_dim=d, budget=B, recent=r, history=w, drop=m))
    seen = []

    def check(s, I, pos, ev):
        n = I.shape[1]
        seen.append(s)
        for u in range(U):
            e = ev[u]
            assert np.all(np.diff(e) > 0), "evicted slots must be ascending and distinct"
            assert e.max() < n - r, "a slot of the recent window was evicted"
            keep_c = np.setdiff1d(np.arange(n - r), e)
            assert I[u, e].min() >= I[u, keep_c].max(), "a surviving candidate outranks an evicted one"
            # brute force: among all m-subsets of the candidates, the evicted one has the
            # largest total record, and is the lexicographically smallest such subset
            best, best_sum = None, -1
            for sub in itertools.combinations(range(n - r), m):
                tot = int(I[u, list(sub)].sum())
                if tot > best_sum:
                    best, best_sum = sub, tot
            assert tuple(e.tolist()) == best

    _run(o, q, k, v, on_compress=check)
    assert len(seen) >= 10


def test_compaction_keeps_order_and_rows():
    rng = np.random.default_rng(7)
    B, r, w, m = 12, 2, 6, 4
    U, T, d = 2, 50, 8
    q, k, v = _rand(rng, U, T, d)
    o = Oracle(_cfg(heads=U, head_dim=d, budget=B, recent=r, history=w, drop=m))
    for s in range(T):
        _, _, due = o.step(q[:, s], k[:, s], v[:, s])
        if due:
            pos0 = o.positions()
            I0 = o.importance()
            ev = o.compress()
            pos1 = o.positions()
            I1 = o.importance()
            K1, V1 = o.rows()
            for u in range(U):
                keep = np.setdiff1d(np.arange(pos0.shape[1]), ev[u])
                assert np.array_equal(pos1[u], pos0[u, keep])
                assert np.all(np.diff(pos1[u]) > 0)
                # every per-row state travels with its row: keys, values, the record
                assert np.array_equal(K1[u], k[u, pos1[u]])
                assert np.array_equal(V1[u], v[u, pos1[u]])
                assert np.array_equal(I1[u], I0[u, keep])
    assert o.n < B + 1


# --------------------------------------------------------------------------------------
# Proof of Lemma A.4: for surviving rows the budgeted weight equals the full-cache weight
# renormalised over the survivors, alpha~_j - beta_j = alpha~_j * sum_{i dropped} beta_i,
# and || a~ - b ||_2 <= 2 * max_j ||v_j||_2 * sum_{j dropped} beta_j.
# --------------------------------------------------------------------------------------
def test_restricted_softmax_identity_against_shadow_full_cache():
    rng = np.random.default_rng(8)
    U, T, d = 3, 80, 16
    q, k, v = _rand(rng, U, T, d)
    o = Oracle(_cfg(heads=U, head_dim=d, budget=20, recent=4, history=8, drop=8))
    k64, v64, q64 = (a.astype(np.float64) for a in (k, v, q))
    dropped_any = False
    for s in range(T):
        out, probs, due = o.step(q[:, s], k[:, s], v[:, s])
        pos = o.positions()
        for u in range(U):
            lg = (k64[u, : s + 1] @ q64[u, s]) / np.sqrt(d)
            beta = np.exp(lg - lg.max())
            beta /= beta.sum()
            S = pos[u]
            gone = np.setdiff1d(np.arange(s + 1), S)
            dropped_any |= gone.size > 0
            a_t = probs[u, : S.size]
            np.testing.assert_allclose(a_t, beta[S] / beta[S].sum(), rtol=1e-11, atol=1e-300)
            np.testing.assert_allclose(a_t - beta[S], a_t * beta[gone].sum(), rtol=1e-7, atol=1e-14)
            b_full = beta @ v64[u, : s + 1]
            bound = 2.0 * np.linalg.norm(v64[u, : s + 1], axis=1).max() * beta[gone].sum()
            assert np.linalg.norm(out[u] - b_full) <= bound + 1e-12
        if due:
            o.compress()
    assert dropped_any


# --------------------------------------------------------------------------------------
# Alg. 2 importance record: counts of "probability < 1/t" over the last w steps.
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("thresh", [sco.INV_POS, sco.INV_LEN])
def test_record_equals_independent_recount_from_probabilities(thresh):
    """Recount the record from the returned probabilities with a different data structure
    (per-position step lists instead of per-slot rings) and compare at every step."""
    rng = np.random.default_rng(9)
    B, r, w, m = 14, 3, 6, 3
    U, T, d = 2, 64, 8
    q, k, v = _rand(rng, U, T, d)
    q *= 2.0
    o = Oracle(_cfg(heads=U, head_dim=d, budget=B, recent=r, history=w, drop=m, thresh_mode=thresh))
    low_steps = [dict() for _ in range(U)]  # position -> list of steps at which it was low
    for s in range(T):
        _, probs, due = o.step(q[:, s], k[:, s], v[:, s])
        t = s + 1
        pos = o.positions()
        n = pos.shape[1]
        tau = np.float32(1.0) / np.float32(t if thresh == sco.INV_POS else n)
        I = o.importance()
        for u in range(U):
            for j in range(n):
                if np.float32(probs[u, j]) < tau:
                    low_steps[u].setdefault(int(pos[u, j]), []).append(t)
            for j in range(n):
                cnt = sum(1 for x in low_steps[u].get(int(pos[u, j]), []) if x > t - w)
                assert I[u, j] == cnt
                age = t - int(pos[u, j])
                assert 0 <= I[u, j] <= min(w, age)
        if due:
            o.compress()


def test_identical_keys_give_zero_record_and_fifo_eviction():
    """All keys equal => every weight is 1/n >= 1/t => no row is ever low => the record is
    zero, the selection is pure tie-break (lowest slots first) and the cache degenerates
    to a sliding window of the newest rows."""
    U, T, d = 2, 60, 8
    B, r, w, m = 9, 2, 4, 3
    rng = np.random.default_rng(10)
    q = rng.standard_normal((U, T, d)).astype(np.float32)
    k = np.broadcast_to(rng.standard_normal((U, 1, d)).astype(np.float32), (U, T, d)).copy()
    v = rng.standard_normal((U, T, d)).astype(np.float32)
    o = Oracle(_cfg(heads=U, head_dim=d, budget=B, recent=r, history=w, drop=m))
    for s in range(T):
        out, probs, due = o.step(q[:, s], k[:, s], v[:, s])
        n = o.n
        np.testing.assert_allclose(probs[:, :n], 1.0 / n, rtol=1e-13)
        assert np.all(o.importance() == 0)
        if due:
            ev = o.compress()
            assert np.array_equal(ev, np.tile(np.arange(m, dtype=np.int32), (U, 1)))
        pos = o.positions()
        assert np.array_equal(pos, np.tile(np.arange(s + 1 - o.n, s + 1), (U, 1)))


def test_dominant_key_survives_and_others_saturate():
    """One key far above the rest => it is never low (record 0) and, once outside the
    recent window, survives every compression; every other row is low at every step it is
    resident, so its record is min(w, age)."""
    U, T, d = 1, 70, 8
    B, r, w, m = 12, 3, 5, 4
    rng = np.random.default_rng(11)
    q = np.zeros((U, T, d), np.float32)
    q[..., 0] = 30.0
    k = 0.01 * rng.standard_normal((U, T, d)).astype(np.float32)
    dom = 0
    k[:, dom, 0] = 10.0
    v = rng.standard_normal((U, T, d)).astype(np.float32)
    o = Oracle(_cfg(heads=U, head_dim=d, budget=B, recent=r, history=w, drop=m))
    for s in range(T):
        out, probs, due = o.step(q[:, s], k[:, s], v[:, s])
        t = s + 1
        pos = o.positions()[0]
        I = o.importance()[0]
        if s >= dom:
            assert dom in pos
            j = int(np.where(pos == dom)[0][0])
            assert I[j] == 0
            others = np.arange(pos.size) != j
            assert np.array_equal(I[others], np.minimum(w, t - pos[others]))
            np.testing.assert_allclose(out[0], v[0, dom], atol=1e-6)
        if due:
            o.compress()
    assert dom in o.positions()[0]


def test_threshold_is_strict_and_uses_tokens_seen():
    """Equal keys and no eviction yet: n = t rows, each weight exactly 1/t, i.e. exactly on
    the threshold (Sec. 3.1: above 1/t counts as significant).  Strict '<' must not flag
    them, for any t (1/t in fp32 equals the fp32 rounding of the double 1/t)."""
    U, d = 1, 4
    o = Oracle(_cfg(heads=1, head_dim=d, budget=64, recent=1, history=64, drop=1))
    one = np.ones((U, d), np.float32)
    for s in range(33):
        o.step(one, one, one)
        assert np.all(o.importance() == 0)


def test_forced_probabilities_drive_only_the_record():
    rng = np.random.default_rng(12)
    U, T, d = 2, 10, 8
    q, k, v = _rand(rng, U, T, d)
    a = Oracle(_cfg(heads=U, head_dim=d, budget=32, history=16))
    b = Oracle(_cfg(heads=U, head_dim=d, budget=32, history=16))
    for s in range(T):
        forced = np.zeros((U, 40), np.float32)  # everything "low"
        forced[:, 0] = 1.0  # except slot 0
        oa, pa, _ = a.step(q[:, s], k[:, s], v[:, s])
        ob, pb, _ = b.step(q[:, s], k[:, s], v[:, s], p_forced=forced)
        assert np.array_equal(oa, ob) and np.array_equal(pa, pb)
    Ib = b.importance()
    assert np.all(Ib[:, 0] == 0)
    assert np.array_equal(Ib[:, 1:], np.tile(T - np.arange(1, T), (U, 1)))


# --------------------------------------------------------------------------------------
# 4-bit storage (Table 3 names it; the scheme is this repository's: asymmetric, group 64).
# --------------------------------------------------------------------------------------
def test_half_converters_match_numpy():
    l = sco.lib()
    bits = np.arange(0, 65536, 7, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([l.sco_half_to_float(int(b)) for b in bits], np.float32)
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok].view(np.uint32), got[ok].view(np.uint32))
    rng = np.random.default_rng(13)
    x = np.concatenate([rng.standard_normal(3000).astype(np.float32) * s
                        for s in (1, 1e-3, 1e-5, 1e-7, 3e-8, 100, 3e4)])
    x = np.concatenate([x, np.float32([0.0, -0.0, 65504, 65519.9, 2 ** -24, 2 ** -25, 1.5 * 2 ** -24,
                                       2.5 * 2 ** -24, 1 + 2 ** -11, 1 + 3 * 2 ** -11])])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([l.sco_float_to_half(float(f)) for f in x], np.uint16)
    assert np.array_equal(want, got)


@pytest.mark.parametrize("d", [64, 128])
def test_int4_storage_round_trip(d):
    rng = np.random.default_rng(14)
    for trial in range(50):
        x = (rng.standard_normal(d) * rng.choice([0.01, 1.0, 30.0])).astype(np.float16)
        if trial == 0:
            x[:64] = np.float16(0.75)  # constant group: range 0 -> scale 1, all codes 0
        codes, scale, zero, stored = sco.i4_roundtrip(x)
        assert codes.min() >= 0 and codes.max() <= 15
        xf = x.astype(np.float32)
        for g in range(d // 64):
            sl = slice(64 * g, 64 * g + 64)
            assert zero[g] == xf[sl].min()
            rng_g = float(xf[sl].max()) - float(xf[sl].min())
            if rng_g == 0:
                assert scale[g] == 1.0 and np.all(codes[sl] == 0)
                assert np.array_equal(stored[sl], xf[sl])
                continue
            s = float(scale[g])
            assert abs(s - rng_g / 15) <= 2 ** -11 * (rng_g / 15) * 1.0001  # fp16 rounding of the step
            assert codes[sl][np.argmin(xf[sl])] == 0
            assert codes[sl][np.argmax(xf[sl])] == 15
            # reconstruction: value = code*scale + zero, within half a step of the input
            # except where the clamp at 15 bites because the fp16 step was rounded down
            np.testing.assert_allclose(stored[sl], codes[sl] * np.float32(s) + np.float32(zero[g]),
                                       rtol=1e-6, atol=1e-7)
            err = np.abs(stored[sl].astype(np.float64) - xf[sl])
            slack = 15 * abs(s - rng_g / 15)
            assert err.max() <= s / 2 + slack + 1e-6 * max(1.0, abs(float(zero[g])))
            # codes are the nearest integer of (x - zero)/scale
            ideal = np.clip(np.rint((xf[sl].astype(np.float64) - float(zero[g])) / s), 0, 15)
            frac = (xf[sl].astype(np.float64) - float(zero[g])) / s
            near_half = np.abs(frac - np.floor(frac) - 0.5) < 1e-4
            assert np.array_equal(codes[sl][~near_half], ideal[~near_half].astype(np.uint8))


def test_int4_cache_attends_over_stored_values():
    """With budget >= length the int4 cache is textbook attention over the *stored* rows."""
    rng = np.random.default_rng(15)
    U, T, d = 2, 12, 64
    q, k, v = _rand(rng, U, T, d, np.float16)
    o = Oracle(_cfg(heads=U, head_dim=d, kv_dtype=sco.I4G64, budget=32, history=8))
    for s in range(T):
        out, probs, _ = o.step(q[:, s], k[:, s], v[:, s])
    Ks, Vs = o.rows()
    for u in range(U):
        for j in range(T):
            assert np.array_equal(Ks[u, j], sco.i4_roundtrip(k[u, j])[3])
            assert np.array_equal(Vs[u, j], sco.i4_roundtrip(v[u, j])[3])
        lg = torch.from_numpy(Ks[u].astype(np.float64) @ q[u, T - 1].astype(np.float64) / np.sqrt(d))
        p = torch.softmax(lg, 0).numpy()
        np.testing.assert_allclose(probs[u, :T], p, rtol=1e-12)
        np.testing.assert_allclose(out[u], p @ Vs[u].astype(np.float64), rtol=1e-11, atol=1e-13)


# --------------------------------------------------------------------------------------
# Record mode "recompute": Alg. 2 as printed collects the record at compression time with an
# extra attention computation over the history window (Sec. 4.1, "Overhead Tradeoff").
# --------------------------------------------------------------------------------------
def _recompute_cfg(**kw):
    return _cfg(record_mode=sco.RECORD_RECOMPUTE, **kw)


@pytest.mark.parametrize("thresh", [sco.INV_POS, sco.INV_LEN])
def test_recompute_equals_online_until_the_first_eviction(thresh):
    """Before anything has been evicted the rows resident now that step i could see are the
    rows step i did see, so replaying its attention changes nothing: the recomputed record is
    the online record, at every step up to and including the first compression."""
    rng = np.random.default_rng(21)
    U, d, B, r, w, m = 3, 16, 14, 2, 6, 4
    T = B + 1
    q, k, v = _rand(rng, U, T, d)
    q *= 2.5
    o = Oracle(_recompute_cfg(heads=U, head_dim=d, budget=B, recent=r, history=w, drop=m,
                              thresh_mode=thresh))
    for s in range(T):
        _, _, due = o.step(q[:, s], k[:, s], v[:, s])
        assert np.array_equal(o.importance(), o.importance_online()), "step %d" % s
        assert o.importance().max() > 0 or s < 3
    assert due
    online = o.importance_online()
    ev, probs, rec = o.compress_recompute()
    assert np.array_equal(rec, online)


def test_recompute_with_window_of_one_is_the_online_record():
    """With w = 1 only the current step is replayed, over exactly the rows it has just
    attended over: both record modes coincide at every compression, also after evictions."""
    rng = np.random.default_rng(22)
    U, d, B, r, m = 2, 8, 9, 2, 3
    T = 40
    q, k, v = _rand(rng, U, T, d)
    q *= 3.0
    o = Oracle(_recompute_cfg(heads=U, head_dim=d, budget=B, recent=r, history=1, drop=m))
    seen = 0
    for s in range(T):
        _, _, due = o.step(q[:, s], k[:, s], v[:, s])
        if due:
            online = o.importance_online()
            _, _, rec = o.compress_recompute()
            assert np.array_equal(rec, online)
            seen += 1
    assert seen >= 5


def test_recompute_probabilities_are_full_attention_restricted_to_the_survivors():
    """Restricted-softmax identity used in the proof of Lemma A.4: the replayed attention of
    step i over the rows that survive is the full-attention distribution of step i restricted
    to those rows and renormalised.  The full-attention side comes from a shadow cache that
    never evicts (pinned above against a library softmax).  The record then follows from
    those probabilities and the threshold 1/i; rows born after step i are not seen by it."""
    rng = np.random.default_rng(23)
    U, d, B, r, w, m = 2, 16, 12, 3, 7, 4
    T = 60
    q, k, v = _rand(rng, U, T, d)
    q *= 2.0
    o = Oracle(_recompute_cfg(heads=U, head_dim=d, budget=B, recent=r, history=w, drop=m))
    full = Oracle(_cfg(heads=U, head_dim=d, budget=T, recent=r, history=w, drop=m))
    beta = []  # beta[s][u, :s+1]: full attention of step s+1 over all tokens
    compressions = 0
    for s in range(T):
        _, _, due = o.step(q[:, s], k[:, s], v[:, s])
        _, pf, _ = full.step(q[:, s], k[:, s], v[:, s])
        beta.append(pf[:, : s + 1].copy())
        if not due:
            continue
        t = s + 1
        pos = o.positions()
        n = o.n
        ev, probs, rec = o.compress_recompute()
        W = min(w, t)
        want = np.zeros((U, n), dtype=np.int64)
        for kk in range(W):
            i = t - W + 1 + kk
            for u in range(U):
                vis = pos[u] <= i - 1
                assert vis.any()
                b = beta[i - 1][u][pos[u][vis]]
                np.testing.assert_allclose(probs[u, kk, :n][vis], b / b.sum(), rtol=1e-9)
                assert np.all(probs[u, kk, :n][~vis] == 0.0)
                low = probs[u, kk, :n].astype(np.float32) < np.float32(1.0) / np.float32(i)
                want[u] += low & vis
        assert np.array_equal(rec, want)
        compressions += 1
    assert compressions >= 8


def test_recompute_forced_probabilities_drive_only_the_record():
    rng = np.random.default_rng(24)
    U, d, B, r, w, m = 2, 8, 9, 2, 4, 3
    q, k, v = _rand(rng, U, B + 1, d)
    o = Oracle(_recompute_cfg(heads=U, head_dim=d, budget=B, recent=r, history=w, drop=m))
    for s in range(B + 1):
        o.step(q[:, s], k[:, s], v[:, s])
    forced = np.ones((U, w, B + 1), dtype=np.float32)   # nothing is low ...
    forced[:, :, 5] = 0.0                                # ... except slot 5, for every replayed step
    ev, probs, rec = o.compress_recompute(p_forced=forced)
    assert np.all(rec[:, 5] == w) and rec.sum() == U * w
    assert np.array_equal(ev, np.array([[0, 1, 5]] * U))  # the largest record, then ties by age
    assert np.all(np.abs(probs.sum(axis=2) - 1.0) < 1e-12)  # the oracle's own probabilities are untouched


# --------------------------------------------------------------------------------------
# Diagnostics the paper plots (oracle/diag.py): persistence ratio (Sec. 3.1) and the
# attention-score change ratio (Sec. 5), pinned on closed forms produced by the oracle cache.
# --------------------------------------------------------------------------------------
def _full_attention_rows(q, k):
    """Probabilities of every position of one unit from a cache that never evicts."""
    T, d = q.shape
    o = Oracle(_cfg(heads=1, head_dim=d, budget=T, recent=1, history=1, drop=1))
    rows = []
    for s in range(T):
        _, p, _ = o.step(q[None, s], k[None, s], np.zeros((1, d), np.float32))
        rows.append(p[0, : s + 1].copy())
    return rows


def test_persistence_counts_on_closed_forms():
    from oracle import diag
    rng = np.random.default_rng(31)
    T, d, split = 24, 8, 12
    e0 = np.zeros(d, np.float32)
    e0[0] = 1.0
    # (a) one dominant token: every position gives token 0 far more than the average share, every
    # other token far less -> both pivotal sets are {0}, ratio 1
    k = rng.standard_normal((T, d)).astype(np.float32) * 0.01
    k[0] += 40.0 * e0
    q = np.tile(8.0 * e0, (T, 1)).astype(np.float32)
    assert diag.persistence_counts(_full_attention_rows(q, k), split) == (1, 1, 1)
    # (b) every position attends to itself only: S_first is every token but the very first
    # (alone in its row it holds exactly 1/t = 1, not more), and nothing persists
    eye = 30.0 * np.eye(T, d * 3, dtype=np.float32)
    rows = _full_attention_rows(eye, eye)
    assert diag.persistence_counts(rows, split) == (split - 1, 0, 0)
    # (c) identical keys: every score is exactly the average, never above it
    one = np.ones((T, d), np.float32)
    assert diag.persistence_counts(_full_attention_rows(one, one), split) == (0, 0, 0)
    # (d) the sets only ever hold tokens below the split, and S_first only needs the first rows
    q, k = (rng.standard_normal((T, d)).astype(np.float32) * 2 for _ in range(2))
    rows = _full_attention_rows(q, k)
    first, later = diag.pivotal_sets(rows, split)
    assert all(j < split for j in first | later)
    assert first == diag.pivotal_sets(rows[:split], split)[0]


def test_change_ratio_of_survivors_is_one_over_kept_mass_minus_one():
    """Sec. 5 defines the change ratio (a_s - a_o)/a_o; with the restricted-softmax identity of
    Lemma A.4 it is the same number for every surviving token of a step, 1/mass - 1 with
    mass the full attention the survivors hold, and -1 for every evicted token."""
    from oracle import diag
    rng = np.random.default_rng(32)
    U, d, B, r, w, m = 2, 16, 12, 3, 6, 4
    T = 50
    q, k, v = _rand(rng, U, T, d)
    q *= 2.0
    o = Oracle(_cfg(heads=U, head_dim=d, budget=B, recent=r, history=w, drop=m))
    full = Oracle(_cfg(heads=U, head_dim=d, budget=T, recent=r, history=w, drop=m))
    for s in range(T):
        _, ps, due = o.step(q[:, s], k[:, s], v[:, s])
        _, pf, _ = full.step(q[:, s], k[:, s], v[:, s])
        pos = o.positions()
        n = o.n
        for u in range(U):
            mass = diag.kept_mass(pos[u], pf[u])
            assert 0.0 < mass <= 1.0 + 1e-12
            ratio = diag.change_ratio(ps[u, :n], pf[u][pos[u]])
            np.testing.assert_allclose(ratio, 1.0 / mass - 1.0, rtol=1e-8, atol=1e-10)
            gone = np.setdiff1d(np.arange(s + 1), pos[u])
            assert np.all(diag.change_ratio(np.zeros(len(gone)), pf[u][gone]) == -1.0)
        if due:
            o.compress()
