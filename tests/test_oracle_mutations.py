"""The pins must be able to fail: plant plausible mistakes in copies of the oracle (on the CPU,
in a temporary directory) and check that at least one pin catches each of them.

Each mutation is a textual edit of ``oracle/sco.c`` compiled into its own shared library; a
reduced version of the pins from ``test_oracle_pins.py`` is run against it in-process through
a second ``ctypes`` handle.  A mutation that no check notices would mean the pins leave that
part of the oracle unpinned.
"""
import ctypes as C
import itertools
import os
import subprocess

import numpy as np
import pytest

from oracle import sco

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "sco.c")

MUTATIONS = {
    "score-sign": ("s[j] = h->scale * acc;", "s[j] = -h->scale * acc;"),
    "no-scale": ("s[j] = h->scale * acc;", "s[j] = acc;"),
    "softmax-no-max-shift-wrong-denominator": ("denom += s[j];", "denom += s[j] * (j ? 1.0 : 0.5);"),
    "value-index-transposed": ("o[ch] += s[j] * (double)V[(size_t)j * d + ch];",
                               "o[ch] += s[j] * (double)V[(size_t)j * d + (d - 1 - ch)];"),
    "key-used-as-value": ("o[ch] += s[j] * (double)V[(size_t)j * d + ch];",
                          "o[ch] += s[j] * (double)K[(size_t)j * d + ch];"),
    "self-row-excluded": ("attention_probabilities(h, K, n, qd, s); /* s now",
                          "attention_probabilities(h, K, n - 1 + (n == 1), qd, s); s[n - 1] = n == 1 ? s[0] : 0.0; /* s now"),
    "threshold-not-strict": ("(uint8_t)(pj < c->tau)", "(uint8_t)(pj <= c->tau)"),
    "threshold-on-length": ("1.0f / (float)c.n_after : 1.0f / (float)c.t_after",
                            "1.0f / (float)c.n_after : 1.0f / (float)c.n_after"),
    "window-one-too-long": ("int ring = (int)(c->t_after % w);", "int ring = (int)(c->t_after % (w + 1) % w);"),
    "new-row-inherits-flags": ("memset(low + (size_t)slot * w, 0, (size_t)w);", ""),
    "recent-window-ignored": ("const int ncand = n - h->r;", "const int ncand = n;"),
    "evict-smallest-record": ("if (best < 0 || I[j] > I[best]) best = j;",
                              "if (best < 0 || I[j] < I[best]) best = j;"),
    "ties-take-highest-slot": ("if (best < 0 || I[j] > I[best]) best = j;",
                               "if (best < 0 || I[j] >= I[best]) best = j;"),
    "flags-left-behind": ("memcpy(low + (size_t)dst * w, low + (size_t)j * w, (size_t)w);", ""),
    "values-left-behind": ("memcpy(V + (size_t)dst * d, V + (size_t)j * d, sizeof(float) * (size_t)d);", ""),
    "drops-one-too-few": ("h->n -= h->m;", "h->n -= h->m - (h->m > 1);"),
    "trigger-at-budget": ("c->budget + 1;", "c->budget;"),
    "int4-truncates": ("float rq = nearbyintf(qv);", "float rq = floorf(qv);"),
    "int4-scale-from-max": ("volatile float range = mx - mn;", "volatile float range = mx;"),
    # record mode "recompute"
    "replay-sees-one-future-row": ("while (vis < n && pos[vis] <= i - 1) ++vis;",
                                   "while (vis < n && pos[vis] <= i) ++vis;"),
    "replay-threshold-uses-current-step": ("1.0f / (float)vis : 1.0f / (float)i;",
                                           "1.0f / (float)vis : 1.0f / (float)h->t;"),
    "replay-window-off-by-one": ("const int64_t i = h->t - W + 1 + k;", "const int64_t i = h->t - W + k;"),
    "replay-wrong-query": ("const float *q = h->Qh + ((size_t)u * w + (size_t)(i % w)) * d;",
                           "const float *q = h->Qh + ((size_t)u * w + (size_t)((i + 1) % w)) * d;"),
    "query-not-kept": ("qkeep[ch] = (float)qd[ch];", "qkeep[ch] = 0.0f;"),
    "replay-counts-invisible-rows": ("for (int j = 0; j < vis; ++j) {\n            const double p = s[j];",
                                     "for (int j = 0; j < n; ++j) {\n            const double p = j < vis ? s[j] : 0.0;"),
}


def _build(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation anchor for %s must occur exactly once" % name
    src = tmp_path / ("sco_%s.c" % name)
    src.write_text(text.replace(old, new))
    lib = tmp_path / ("libsco_%s.so" % name)
    subprocess.run(["gcc", "-std=c11", "-O1", "-ffp-contract=off", "-fPIC", "-shared", "-pthread", "-w",
                    "-o", str(lib), str(src), "-lm"], check=True)
    return str(lib)


class _Cache:
    """Minimal driver of a (possibly mutated) oracle library."""

    def __init__(self, lib, heads, d, kv, B, r, w, m, trigger=0, thresh=0, record_mode=0):
        self.l = C.CDLL(lib)
        self.l.sco_create.restype = C.c_void_p
        cfg = sco._Cfg(1, heads, d, kv, B, r, w, m, trigger, thresh, 0.0, record_mode)
        self.h = C.c_void_p(self.l.sco_create(C.byref(cfg), 1))
        assert self.h
        self.U, self.d, self.m = heads, d, m
        n, t, cap = C.c_int32(), C.c_int64(), C.c_int32()
        self.l.sco_len(self.h, C.byref(n), C.byref(t), C.byref(cap))
        self.cap = cap.value
        self.dt = np.float32 if kv == sco.F32 else np.float16

    def n(self):
        n = C.c_int32()
        self.l.sco_len(self.h, C.byref(n), None, None)
        return n.value

    def step(self, q, k, v):
        q, k, v = (np.ascontiguousarray(a, dtype=self.dt) for a in (q, k, v))
        out = np.zeros((self.U, self.d))
        probs = np.zeros((self.U, self.cap))
        due = C.c_int32()
        p = lambda a: a.ctypes.data_as(C.c_void_p)
        assert self.l.sco_step(self.h, p(q), p(k), p(v), p(out), p(probs), None, 0, C.byref(due)) == 0
        return out, probs, bool(due.value)

    def importance(self):
        I = np.zeros((self.U, self.n()), np.int32)
        self.l.sco_importance(self.h, I.ctypes.data_as(C.c_void_p))
        return I

    def positions(self):
        P = np.zeros((self.U, self.n()), np.int64)
        self.l.sco_positions(self.h, P.ctypes.data_as(C.c_void_p))
        return P

    def rows(self):
        n = self.n()
        K = np.zeros((self.U, n, self.d), np.float32)
        V = np.zeros((self.U, n, self.d), np.float32)
        self.l.sco_rows(self.h, K.ctypes.data_as(C.c_void_p), V.ctypes.data_as(C.c_void_p))
        return K, V

    def compress(self):
        ev = np.zeros((self.U, self.m), np.int32)
        assert self.l.sco_compress(self.h, ev.ctypes.data_as(C.c_void_p)) == 0
        return ev

    def importance_online(self):
        I = np.zeros((self.U, self.n()), np.int32)
        self.l.sco_importance_online(self.h, I.ctypes.data_as(C.c_void_p))
        return I

    def compress_recompute(self, W):
        n = self.n()
        ev = np.zeros((self.U, self.m), np.int32)
        probs = np.zeros((self.U, W, self.cap))
        rec = np.zeros((self.U, n), np.int32)
        p = lambda a: a.ctypes.data_as(C.c_void_p)
        assert self.l.sco_compress_recompute(self.h, p(ev), p(probs), None, 0, p(rec)) == 0
        return ev, probs, rec


def _pins(lib):
    """A condensed run of the pins; raises AssertionError when one of them fails."""
    rng = np.random.default_rng(0)
    # (1) budget >= length: textbook attention (numpy), probabilities sum to one
    U, T, d = 2, 24, 8
    q, k, v = (rng.standard_normal((U, T, d)).astype(np.float32) for _ in range(3))
    c = _Cache(lib, U, d, sco.F32, T, 2, 6, 3)
    for s in range(T):
        out, probs, due = c.step(q[:, s], k[:, s], v[:, s])
        lg = np.einsum("ud,utd->ut", q[:, s].astype(np.float64), k[:, : s + 1].astype(np.float64)) / np.sqrt(d)
        p = np.exp(lg - lg.max(1, keepdims=True))
        p /= p.sum(1, keepdims=True)
        np.testing.assert_allclose(probs[:, : s + 1], p, rtol=1e-10)
        np.testing.assert_allclose(out, np.einsum("ut,utd->ud", p, v[:, : s + 1].astype(np.float64)),
                                   rtol=1e-9, atol=1e-12)
        assert due == (s == T - 1 and False) or not due or s == T - 1
    # (2) compression: sizes, recent window, brute force, record recount, row integrity, identity
    B, r, w, m = 10, 3, 5, 3
    T = 48
    q, k, v = (rng.standard_normal((U, T, d)).astype(np.float32) for _ in range(3))
    q *= 3.0
    c = _Cache(lib, U, d, sco.F32, B, r, w, m)
    low_steps = [dict() for _ in range(U)]
    for s in range(T):
        out, probs, due = c.step(q[:, s], k[:, s], v[:, s])
        t = s + 1
        n = c.n()
        assert due == (n == B + 1)
        pos = c.positions()
        I = c.importance()
        K, V = c.rows()
        tau = np.float32(1.0) / np.float32(t)
        for u in range(U):
            assert np.array_equal(K[u], k[u, pos[u]]) and np.array_equal(V[u], v[u, pos[u]])
            lg = (k[u, : s + 1].astype(np.float64) @ q[u, s].astype(np.float64)) / np.sqrt(d)
            beta = np.exp(lg - lg.max())
            beta /= beta.sum()
            np.testing.assert_allclose(probs[u, :n], beta[pos[u]] / beta[pos[u]].sum(), rtol=1e-9)
            for j in range(n):
                if np.float32(probs[u, j]) < tau:
                    low_steps[u].setdefault(int(pos[u, j]), []).append(t)
                assert I[u, j] == sum(1 for x in low_steps[u].get(int(pos[u, j]), []) if x > t - w)
        if due:
            ev = c.compress()
            assert c.n() == B + 1 - m
            for u in range(U):
                assert ev[u].max() < n - r
                best, best_sum = None, -1
                for sub in itertools.combinations(range(n - r), m):
                    tot = int(I[u, list(sub)].sum())
                    if tot > best_sum:
                        best, best_sum = sub, tot
                assert tuple(ev[u].tolist()) == best
    # (2b) record mode "recompute": equal to the online record while nothing has been evicted;
    # afterwards the replayed probabilities are full attention restricted to the survivors
    # and the record is their count below 1/i over the rows each replayed step could see
    B, r, w, m = 10, 3, 5, 3
    T = 40
    q, k, v = (rng.standard_normal((U, T, d)).astype(np.float32) for _ in range(3))
    q *= 3.0
    c = _Cache(lib, U, d, sco.F32, B, r, w, m, record_mode=1)
    evicted_yet = False
    for s in range(T):
        out, probs, due = c.step(q[:, s], k[:, s], v[:, s])
        t = s + 1
        if not evicted_yet:
            assert np.array_equal(c.importance(), c.importance_online())
        if due:
            pos = c.positions()
            n = c.n()
            W = min(w, t)
            ev, pr, rec = c.compress_recompute(W)
            want = np.zeros((U, n), np.int64)
            for kk in range(W):
                i = t - W + 1 + kk
                for u in range(U):
                    vis = pos[u] <= i - 1
                    lg = (k[u, :i].astype(np.float64) @ q[u, i - 1].astype(np.float64)) / np.sqrt(d)
                    beta = np.exp(lg - lg.max())
                    b = beta[pos[u][vis]]
                    np.testing.assert_allclose(pr[u, kk, :n][vis], b / b.sum(), rtol=1e-9)
                    assert np.all(pr[u, kk, :n][~vis] == 0.0)
                    want[u] += (pr[u, kk, :n].astype(np.float32) < np.float32(1.0) / np.float32(i)) & vis
            assert np.array_equal(rec, want)
            evicted_yet = True
    # (3) identical keys: nothing is ever low (strict threshold on 1/t)
    c = _Cache(lib, 1, 4, sco.F32, 64, 1, 64, 1)
    one = np.ones((1, 4), np.float32)
    for s in range(20):
        c.step(one, one, one)
        assert np.all(c.importance() == 0)
    # (4) int4 storage: min and max of a group map to codes 0 and 15, error within half a step
    x = (rng.standard_normal(64) * 2).astype(np.float16)
    l = C.CDLL(lib)
    codes = np.zeros(64, np.uint8)
    sc_, ze = np.zeros(1, np.float16), np.zeros(1, np.float16)
    st = np.zeros(64, np.float32)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    assert l.sco_i4_roundtrip(p(x), 64, p(codes), p(sc_), p(ze), p(st)) == 0
    xf = x.astype(np.float32)
    assert codes[np.argmin(xf)] == 0 and codes[np.argmax(xf)] == 15
    step = (float(xf.max()) - float(xf.min())) / 15
    assert abs(float(sc_[0]) - step) <= 2 ** -11 * step * 1.001
    assert np.abs(st - xf).max() <= float(sc_[0]) * 0.5 + 15 * abs(float(sc_[0]) - (xf.max() - xf.min()) / 15) + 1e-6


def test_pins_pass_on_the_real_oracle():
    _pins(sco.build())


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_pins_catch_planted_mistake(name, tmp_path):
    old, new = MUTATIONS[name]
    lib = _build(tmp_path, name, old, new)
    with pytest.raises(AssertionError):
        _pins(lib)
