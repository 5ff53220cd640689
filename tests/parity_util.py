"""Shared driver of the GPU-vs-oracle parity tests.

Protocol (forced-probabilities mode): at every step the GPU library emits `out` and the fp32
probabilities it tested against the threshold; the oracle takes the same inputs plus those
probabilities for its own low-score decision, so the integer side (records, evicted slots,
positions, stored rows) must agree bit for bit, while `out` and the probabilities themselves
are compared with the oracle's double-precision values within the floating-point tolerance.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import sco
from oracle.sco import Oracle, OracleConfig
from paper_2305_17118_amd import binding as B
from paper_2305_17118_amd.workloads import Workload, streams

# spec tolerances: relative error of the attention output
TOL = {B.SC_KV_F32: 1e-5, B.SC_KV_F16: 2e-3, B.SC_KV_I4G64: 2e-3}


def dequant_i4(codes_u8: np.ndarray, meta_f16: np.ndarray) -> np.ndarray:
    """codes [..., d/2] bytes (channel 2i in the low nibble), meta [..., d/64, 2] fp16 (scale, zero)
    -> fp32 [..., d] = code*scale + zero (each a single fp32 operation)."""
    lo = (codes_u8 & 15).astype(np.float32)
    hi = (codes_u8 >> 4).astype(np.float32)
    codes = np.stack([lo, hi], axis=-1).reshape(*codes_u8.shape[:-1], -1)
    d = codes.shape[-1]
    scale = np.repeat(meta_f16[..., 0].astype(np.float32), 64, axis=-1)[..., :d]
    zero = np.repeat(meta_f16[..., 1].astype(np.float32), 64, axis=-1)[..., :d]
    return (codes * scale).astype(np.float32) + zero


def compare_step(o_gpu, o_ref, p_gpu, p_ref, tol, kv_dtype, stats, label):
    """One step's outputs [U, d] and probabilities [U, n] against the oracle's, within the
    spec tolerance; updates the running maxima in `stats`."""
    assert np.all(np.isfinite(o_gpu)) and np.all(np.isfinite(p_gpu)), label
    sum_err = np.abs(p_gpu.astype(np.float64).sum(axis=1) - 1.0).max()
    assert sum_err <= 1e-5, "%s: probabilities sum off by %g" % (label, sum_err)
    dp = np.abs(p_gpu - p_ref).max(axis=1)
    lim = tol * p_ref.max(axis=1) if kv_dtype != B.SC_KV_F32 else 1e-5
    assert np.all(dp <= lim), "%s: probability error %g" % (label, dp.max())
    rel = np.linalg.norm(o_gpu - o_ref, axis=1) / np.linalg.norm(o_ref, axis=1)
    assert np.all(rel <= tol), "%s: output relative error %g > %g" % (label, rel.max(), tol)
    rms = np.sqrt((o_ref ** 2).mean(axis=1, keepdims=True))
    assert np.all(np.abs(o_gpu - o_ref) <= tol * (np.abs(o_ref) + rms)), "%s elementwise" % label
    st = stats
    st["max_rel_out"] = max(st["max_rel_out"], float(rel.max()))
    st["max_dp"] = max(st["max_dp"], float(dp.max()))
    st["max_sum_err"] = max(st["max_sum_err"], float(sum_err))


class ParityRun:
    """One workload on the GPU (all units) and on the oracle (the units in `sel`)."""

    def __init__(self, wl: Workload, sel=None, trigger=B.SC_TRIGGER_HARD_CAP,
                 thresh=B.SC_THRESH_INV_POS, scale=0.0, steps=None, device="cuda:0", qkv=None,
                 window_mode=B.SC_WINDOW_AUTO, record_mode=B.SC_RECORD_ONLINE):
        self.wl = wl
        self.dev = torch.device(device)
        self.U = wl.units
        self.sel = list(range(self.U)) if sel is None else list(sel)
        self.T = wl.total if steps is None else steps
        self.cfg = B.make_config(wl.batch, wl.heads, wl.head_dim, wl.kv_dtype, wl.budget, wl.recent,
                                 wl.history, wl.drop, trigger, thresh, scale, window_mode, record_mode)
        self.recompute = record_mode == B.SC_RECORD_RECOMPUTE
        self.cache = B.BudgetCache(self.cfg, device)
        self.oracle = Oracle(OracleConfig(1, len(self.sel), wl.head_dim, wl.kv_dtype, wl.budget,
                                          wl.recent, wl.history, wl.drop, trigger, thresh, scale,
                                          record_mode))
        q, k, v = qkv if qkv is not None else streams(wl, steps=self.T, threads=16)
        self.hq, self.hk, self.hv = (np.ascontiguousarray(a[self.sel]) for a in (q, k, v))
        self.q, self.k, self.v = (torch.from_numpy(a).to(self.dev) for a in (q, k, v))
        del q, k, v
        self.sel_t = torch.tensor(self.sel, device=self.dev, dtype=torch.long)
        self.out = torch.empty(self.U, wl.head_dim, dtype=self.cache.io_dtype, device=self.dev)
        self.probs = torch.zeros(self.U, self.cache.capacity, dtype=torch.float32, device=self.dev)
        self.evicted = torch.empty(self.U, wl.drop, dtype=torch.int32, device=self.dev)
        self.tol = TOL[wl.kv_dtype]
        self.stats = dict(steps=0, compressions=0, max_rel_out=0.0, max_dp=0.0, max_sum_err=0.0)
        self.step_idx = 0

    # -- one step on both sides, compared ------------------------------------------------
    def step(self, check=True):
        s = self.step_idx
        d = self.wl.head_dim
        stride = self.T * d
        due = self.cache.decode_step(self.q[:, s], self.k[:, s], self.v[:, s], self.out,
                                     self.probs, in_stride=stride)
        n = self.cache.n
        p_gpu = self.probs.index_select(0, self.sel_t)[:, :n].cpu().numpy()
        o_gpu = self.out.index_select(0, self.sel_t).float().cpu().numpy().astype(np.float64)
        o_ref, p_ref, due_ref = self.oracle.step(self.hq[:, s], self.hk[:, s], self.hv[:, s],
                                                 p_forced=p_gpu)
        assert due == due_ref and n == self.oracle.n and self.cache.t == self.oracle.t
        if check:
            self._compare(o_gpu, o_ref, p_gpu, p_ref[:, :n], s)
        self.step_idx += 1
        self.stats["steps"] += 1
        return due

    def _compare(self, o_gpu, o_ref, p_gpu, p_ref, s):
        compare_step(o_gpu, o_ref, p_gpu, p_ref, self.tol, self.wl.kv_dtype, self.stats, "step %d" % s)

    # -- the prompt through sc_prefill, the oracle stepped through the same positions ----------
    def prefill(self, P, mode=B.SC_PREFILL_AUTO):
        """Positions 0..P-1 of the streams go through ONE sc_prefill call; the oracle takes them
        one step at a time with the GPU's probabilities of that position forced, and every
        position's output and probabilities are compared.  Evictions inside the call are not
        visible one by one; the positions and stored rows after the call are, and must agree
        bit for bit (any differing eviction changes them)."""
        s0 = self.step_idx  # the call continues the stream from wherever the cache stands
        d, C = self.wl.head_dim, self.cache.capacity
        out = torch.empty(self.U, P, d, dtype=self.cache.io_dtype, device=self.dev)
        probs = torch.zeros(self.U, P, C, dtype=torch.float32, device=self.dev)
        self.cache.prefill(self.q[:, s0:], self.k[:, s0:], self.v[:, s0:], P, self.T * d, out, probs, mode)
        o_all = out.index_select(0, self.sel_t).float().cpu().numpy().astype(np.float64)
        p_all = probs.index_select(0, self.sel_t).cpu().numpy()
        del out, probs
        for i in range(P):
            s = s0 + i
            n = self.oracle.n + 1
            p_gpu = np.ascontiguousarray(p_all[:, i, :n])
            o_ref, p_ref, due = self.oracle.step(self.hq[:, s], self.hk[:, s], self.hv[:, s],
                                                 p_forced=p_gpu)
            self._compare(o_all[:, i], o_ref, p_gpu, p_ref[:, :n], s)
            self.stats["steps"] += 1
            if due:
                assert not self.recompute, "prefill parity with a recomputed record: step instead"
                self.oracle.compress()
                self.stats["compressions"] += 1
        self.step_idx = s0 + P
        assert (self.cache.n, self.cache.t) == (self.oracle.n, self.oracle.t)
        self.check_state()
        return self.stats

    # -- compression on both sides, integer side bit-exact ---------------------------------
    def gpu_record(self):
        n = self.cache.n
        if self.cache.ring_words:  # exact ring: the record is the popcount of each slot's ring
            ring = self.cache.ring().index_select(0, self.sel_t)[:, :, :n].cpu().numpy()
            bits = np.unpackbits(ring.view(np.uint8).reshape(*ring.shape, 4), axis=-1)
            return bits.sum(axis=(1, 3)).astype(np.int64)
        cnt = self.cache.cnt().index_select(0, self.sel_t)[:, :, :n].to(torch.int32) & 0xFFFF
        return cnt.sum(dim=1).cpu().numpy()

    def compress_recompute(self, check_rows=True):
        """Record mode "recompute": the GPU replays the kept queries inside sc_compress and
        dumps the probabilities its thresholds saw; the oracle replays the same steps with
        those probabilities forced, so the evicted slots must agree bit for bit, and its own
        (double precision) replayed probabilities are compared within tolerance."""
        n, t = self.cache.n, self.cache.t
        W = min(self.wl.history, t)
        probs = torch.zeros(self.U, W, self.cache.capacity, dtype=torch.float32, device=self.dev)
        self.evicted.fill_(-1)
        self.cache.compress(self.evicted, probs)
        p_gpu = probs.index_select(0, self.sel_t)[:, :, :n].cpu().numpy()
        ev_ref, p_ref, rec = self.oracle.compress_recompute(p_forced=p_gpu)
        p_ref = p_ref[:, :, :n]
        assert np.all(np.isfinite(p_gpu))
        seen = p_ref.sum(axis=2) > 0.5  # replayed steps that see at least one resident row
        sum_err = np.abs(p_gpu.astype(np.float64).sum(axis=2) - 1.0)[seen].max()
        assert sum_err <= 1e-5, "replayed probabilities sum off by %g" % sum_err
        assert np.all(p_gpu[~seen] == 0.0)
        dp = np.abs(p_gpu - p_ref).max(axis=2)
        lim = self.tol * p_ref.max(axis=2) if self.wl.kv_dtype != B.SC_KV_F32 else 1e-5
        assert np.all(dp <= lim), "replayed probability error %g" % dp.max()
        ev_gpu = self.evicted.index_select(0, self.sel_t).cpu().numpy()
        assert np.array_equal(ev_gpu, ev_ref), "evicted slots differ"
        self.check_state(check_rows)
        self.stats["compressions"] += 1
        self.stats["max_dp"] = max(self.stats["max_dp"], float(dp.max()))

    def compress(self, check_rows=True):
        if self.recompute:
            return self.compress_recompute(check_rows)
        I_gpu = self.gpu_record()
        I_ref = self.oracle.importance()
        assert np.array_equal(I_gpu, I_ref), "importance records differ before compression %d" % (
            self.stats["compressions"])
        self.evicted.fill_(-1)
        self.cache.compress(self.evicted)
        ev_ref = self.oracle.compress()
        ev_gpu = self.evicted.index_select(0, self.sel_t).cpu().numpy()
        assert np.array_equal(ev_gpu, ev_ref), "evicted slots differ"
        self.check_state(check_rows)
        self.stats["compressions"] += 1

    def check_state(self, check_rows=True):
        n = self.cache.n
        assert n == self.oracle.n
        pos_gpu = self.cache.pos().index_select(0, self.sel_t)[:, :n].cpu().numpy()
        assert np.array_equal(pos_gpu.astype(np.int64), self.oracle.positions()), "positions differ"
        # (the GPU keeps the record in w/m buckets whose union equals the history window only
        # at compression steps, so records are compared there, before each compression)
        # counters of free slots must be clear so that rows appended later start from zero
        planes = self.cache.ring() if self.cache.ring_words else self.cache.cnt()
        tail = planes.index_select(0, self.sel_t)[:, :, n:]
        assert int(tail.abs().max().item()) == 0 if tail.numel() else True
        if not check_rows:
            return
        Kg, Vg = self.cache.kv_rows()
        Kg = Kg.index_select(0, self.sel_t)[:, :n].cpu().numpy()
        Vg = Vg.index_select(0, self.sel_t)[:, :n].cpu().numpy()
        if self.wl.kv_dtype == B.SC_KV_I4G64:
            Km, Vm = self.cache.kv_meta()
            Km = Km.index_select(0, self.sel_t)[:, :n].cpu().numpy()
            Vm = Vm.index_select(0, self.sel_t)[:, :n].cpu().numpy()
            Kg, Vg = dequant_i4(Kg, Km), dequant_i4(Vg, Vm)
        Kr, Vr = self.oracle.rows()
        assert np.array_equal(Kg.astype(np.float32), Kr), "stored K rows differ"
        assert np.array_equal(Vg.astype(np.float32), Vr), "stored V rows differ"

    def run(self, steps=None, check_every=1, check_rows_every=1):
        steps = self.T - self.step_idx if steps is None else steps
        for i in range(steps):
            due = self.step(check=(i % check_every == 0) or i == steps - 1)
            if due:
                self.compress(check_rows=(self.stats["compressions"] % check_rows_every == 0))
        return self.stats
