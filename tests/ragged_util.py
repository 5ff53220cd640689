"""GPU-vs-oracle parity for ragged batches: every sequence has its own prompt length, joins the
decode steps at its own step and leaves after its own number of tokens.  Same protocol as
`parity_util` (the oracle's low-score decision is driven by the GPU's fp32 probabilities, so the
integer side must agree bit for bit), with one single-sequence oracle per batch entry."""
from __future__ import annotations

import numpy as np
import torch

from oracle.ragged import RaggedOracle
from oracle.sco import OracleConfig
from paper_2305_17118_amd import binding as B
from paper_2305_17118_amd.workloads import Workload, streams
from tests.parity_util import TOL, compare_step, dequant_i4


class RaggedParityRun:
    def __init__(self, wl: Workload, prompts, starts, decodes, trigger=B.SC_TRIGGER_HARD_CAP,
                 thresh=B.SC_THRESH_INV_POS, window_mode=B.SC_WINDOW_AUTO,
                 record_mode=B.SC_RECORD_ONLINE, device="cuda:0", check_seqs=None):
        """Sequence b: `prompts[b]` prompt positions (0: none), then `decodes[b]` decode steps
        taken at the global steps starts[b] ... starts[b] + decodes[b] - 1.  `check_seqs`: the
        sequences followed by an oracle (default all); the others run on the GPU only."""
        self.wl = wl
        self.dev = torch.device(device)
        self.batch, self.heads, self.d, self.U = wl.batch, wl.heads, wl.head_dim, wl.units
        assert len(prompts) == len(starts) == len(decodes) == wl.batch
        self.prompts, self.starts, self.decodes = list(prompts), list(starts), list(decodes)
        self.T = max(p + n for p, n in zip(prompts, decodes))
        self.steps_total = max(s + n for s, n in zip(starts, decodes))
        self.cfg = B.make_config(wl.batch, wl.heads, wl.head_dim, wl.kv_dtype, wl.budget, wl.recent,
                                 wl.history, wl.drop, trigger, thresh, 0.0, window_mode, record_mode)
        self.recompute = record_mode == B.SC_RECORD_RECOMPUTE
        self.cache = B.BudgetCache(self.cfg, device)
        self.oracle = RaggedOracle(OracleConfig(wl.batch, wl.heads, wl.head_dim, wl.kv_dtype, wl.budget,
                                                wl.recent, wl.history, wl.drop, trigger, thresh, 0.0,
                                                record_mode))
        q, k, v = streams(wl, steps=self.T, threads=16)
        self.hq, self.hk, self.hv = q, k, v
        self.q, self.k, self.v = (torch.from_numpy(a).to(self.dev) for a in (q, k, v))
        self.C = self.cache.capacity
        self.out = torch.empty(self.U, self.d, dtype=self.cache.io_dtype, device=self.dev)
        self.probs = torch.zeros(self.U, self.C, dtype=torch.float32, device=self.dev)
        self.evicted = torch.empty(self.U, wl.drop, dtype=torch.int32, device=self.dev)
        self.tol = TOL[wl.kv_dtype]
        self.stats = dict(steps=0, seq_steps=0, compressions=0, seq_compressions=0, max_rel_out=0.0,
                          max_dp=0.0, max_sum_err=0.0)
        self.consumed = [0] * self.batch  # stream positions each sequence has taken
        self.check = list(range(self.batch)) if check_seqs is None else sorted(check_seqs)

    def _units(self, b):
        return slice(b * self.heads, (b + 1) * self.heads)

    # -- prompts of different lengths through one sc_prefill_ragged call ---------------------
    def prefill(self, mode=B.SC_PREFILL_AUTO, lengths=None):
        """`lengths` (default: the prompts) more positions per sequence, continuing each
        sequence's stream from the position it has consumed so far."""
        lengths = self.prompts if lengths is None else list(lengths)
        P = max(lengths)
        assert P > 0
        out = torch.full((self.U, P, self.d), float("nan"), dtype=self.cache.io_dtype, device=self.dev)
        probs = torch.zeros(self.U, P, self.C, dtype=torch.float32, device=self.dev)
        # every sequence reads from its own offset: gather the chunks into one [U, P, d] block
        idx = torch.tensor([[min(self.consumed[b] + i, self.T - 1) for i in range(P)]
                            for b in range(self.batch)], device=self.dev).repeat_interleave(self.heads, dim=0)
        ar = torch.arange(self.U, device=self.dev).unsqueeze(1)
        qs, ks, vs = (x[ar, idx].contiguous() for x in (self.q, self.k, self.v))
        self.cache.prefill_ragged(qs, ks, vs, lengths, P * self.d, out, probs, mode)
        for b in range(self.batch):
            if b not in self.check:
                self.consumed[b] += lengths[b]
                continue
            u = self._units(b)
            o_all = out[u].float().cpu().numpy().astype(np.float64)
            p_all = probs[u].cpu().numpy()
            seq = self.oracle.seq[b]
            c0 = self.consumed[b]
            for i in range(lengths[b]):
                s = c0 + i
                n = seq.n + 1
                p_gpu = np.ascontiguousarray(p_all[:, i, :n])
                o_ref, p_ref, due = seq.step(self.hq[u, s], self.hk[u, s], self.hv[u, s], p_forced=p_gpu)
                compare_step(o_all[:, i], o_ref, p_gpu, p_ref[:, :n], self.tol, self.wl.kv_dtype, self.stats,
                             "sequence %d prompt position %d" % (b, s))
                if due:
                    assert not self.recompute, "prefill parity with a recomputed record: step instead"
                    seq.compress()
            # rows past the sequence's own prompt were not written
            assert np.all(np.isnan(o_all[:, lengths[b]:]))
            self.consumed[b] = c0 + lengths[b]
            assert self.cache.len_seq(b) == seq.lengths()[:2]
        del out, probs
        self.check_state()

    def restart(self, b):
        """Sequence b has finished: its slot is emptied for a new request (the other sequences
        keep their state); the oracle side starts a fresh single-sequence oracle."""
        import dataclasses

        from oracle.sco import Oracle

        self.cache.reset_seq(b)
        self.oracle.seq[b] = Oracle(dataclasses.replace(self.oracle.cfg, batch=1))
        assert self.cache.len_seq(b) == (0, 0)

    # -- one ragged decode step ------------------------------------------------------------
    def step(self, s):
        active = [self.starts[b] <= s < self.starts[b] + self.decodes[b] for b in range(self.batch)]
        return self.step_active(active, s)

    def step_active(self, active, s=-1):
        """One decode step of the sequences flagged in `active`, each consuming its next stream
        position."""
        if not any(active):
            return 0
        idx = torch.tensor([self.consumed[b] if active[b] else 0 for b in range(self.batch)],
                           device=self.dev).repeat_interleave(self.heads)
        ar = torch.arange(self.U, device=self.dev)
        qs, ks, vs = (x[ar, idx].contiguous() for x in (self.q, self.k, self.v))
        self.out.fill_(float("nan"))
        self.probs.fill_(-1.0)
        n_due = self.cache.decode_step_ragged(qs, ks, vs, self.out, self.probs, active=active)
        o_gpu = self.out.float().cpu().numpy().astype(np.float64)
        p_gpu = self.probs.cpu().numpy() if len(self.check) == self.batch else None
        n_trig = self.cache.n_trig
        due_ref = 0
        for b in range(self.batch):
            u = self._units(b)
            if not active[b]:  # units of idle sequences are not touched
                assert np.all(np.isnan(o_gpu[u]))
                assert p_gpu is None or np.all(p_gpu[u] == -1.0)
                continue
            if b not in self.check:  # GPU only: its counters still have to follow the schedule
                self.consumed[b] += 1
                due_ref += int(self.cache.len_seq(b)[0] == n_trig)
                self.stats["seq_steps"] += 1
                continue
            seq = self.oracle.seq[b]
            n = seq.n + 1
            i = self.consumed[b]
            pf = (self.probs[u, :n].cpu().numpy() if p_gpu is None else np.ascontiguousarray(p_gpu[u, :n]))
            o_ref, p_ref, due = seq.step(self.hq[u, i], self.hk[u, i], self.hv[u, i], p_forced=pf)
            compare_step(o_gpu[u], o_ref, pf, p_ref[:, :n], self.tol, self.wl.kv_dtype, self.stats,
                         "step %d sequence %d (t=%d)" % (s, b, seq.t))
            self.consumed[b] += 1
            due_ref += int(due)
            assert self.cache.len_seq(b) == seq.lengths()[:2]
            self.stats["seq_steps"] += 1
        assert n_due == due_ref, "step %d: %d sequences due on the GPU, %d on the oracle" % (s, n_due, due_ref)
        self.stats["steps"] += 1
        return n_due

    def gpu_record(self, b, n):
        u = self._units(b)
        if self.cache.ring_words:
            ring = self.cache.ring()[u][:, :, :n].cpu().numpy()
            bits = np.unpackbits(ring.view(np.uint8).reshape(*ring.shape, 4), axis=-1)
            return bits.sum(axis=(1, 3)).astype(np.int64)
        cnt = self.cache.cnt()[u][:, :, :n].to(torch.int32) & 0xFFFF
        return cnt.sum(dim=1).cpu().numpy()

    def compress_recompute(self, due):
        """Record rebuilt at compression time: each due sequence replays its own last min(w, t_b)
        queries; the GPU dumps the probabilities its thresholds saw, the sequence's oracle replays
        the same steps with them forced (evicted slots bit-exact, probabilities within tolerance)."""
        w = self.wl.history
        probs = torch.zeros(self.U, w, self.C, dtype=torch.float32, device=self.dev)
        self.evicted.fill_(-1)
        self.cache.compress_ragged(self.evicted, probs)
        p_all = probs.cpu().numpy()
        ev_gpu = self.evicted.cpu().numpy()
        for b in range(self.batch):
            u = self._units(b)
            if not due[b]:
                assert np.all(ev_gpu[u] == -1) and np.all(p_all[u] == 0.0)  # untouched
                continue
            if b not in self.check:
                continue
            seq = self.oracle.seq[b]
            n, t, _ = seq.lengths()
            W = min(w, t)
            p_gpu = np.ascontiguousarray(p_all[u, :W, :n])
            ev_ref, p_ref, _ = seq.compress_recompute(p_forced=p_gpu)
            p_ref = p_ref[:, :, :n]
            seen = p_ref.sum(axis=2) > 0.5
            assert np.abs(p_gpu.astype(np.float64).sum(axis=2) - 1.0)[seen].max() <= 1e-5
            assert np.all(p_gpu[~seen] == 0.0)
            dp = np.abs(p_gpu - p_ref).max(axis=2)
            lim = self.tol * p_ref.max(axis=2) if self.wl.kv_dtype != B.SC_KV_F32 else 1e-5
            assert np.all(dp <= lim), "sequence %d: replayed probability error %g" % (b, dp.max())
            assert np.array_equal(ev_gpu[u], ev_ref), "sequence %d: evicted slots differ" % b
        self.check_state()
        self.stats["compressions"] += 1
        self.stats["seq_compressions"] += int(due.sum())

    def compress(self):
        n_trig = self.cache.n_trig
        due = np.array([self.cache.len_seq(b)[0] == n_trig for b in range(self.batch)])
        assert due.any() and all(due[b] == self.oracle.due()[b] for b in self.check)
        if self.recompute:
            return self.compress_recompute(due)
        for b in np.flatnonzero(due):
            if b not in self.check:
                continue
            n = self.oracle.seq[b].n
            assert np.array_equal(self.gpu_record(b, n), self.oracle.importance(b)), \
                "sequence %d: importance records differ before its compression" % b
        self.evicted.fill_(-1)
        self.cache.compress_ragged(self.evicted)
        ev_gpu = self.evicted.cpu().numpy()
        for b in range(self.batch):
            u = self._units(b)
            if not due[b]:
                assert np.all(ev_gpu[u] == -1)  # untouched
            elif b in self.check:
                assert np.array_equal(ev_gpu[u], self.oracle.seq[b].compress()), \
                    "sequence %d: evicted slots differ" % b
        self.check_state()
        self.stats["compressions"] += 1
        self.stats["seq_compressions"] += int(due.sum())

    def check_state(self):
        pos = self.cache.pos()
        planes = self.cache.ring() if self.cache.ring_words else self.cache.cnt()
        Kg_all, Vg_all = self.cache.kv_rows()
        for b in self.check:
            u = self._units(b)
            seq = self.oracle.seq[b]
            n, t, _ = seq.lengths()
            assert self.cache.len_seq(b) == (n, t)
            assert np.array_equal(pos[u][:, :n].cpu().numpy().astype(np.int64), seq.positions()), \
                "sequence %d: positions differ" % b
            tail = planes[u][:, :, n:]
            assert int(tail.abs().max().item()) == 0 if tail.numel() else True
            if n == 0:
                continue
            Kg, Vg = Kg_all[u][:, :n].cpu().numpy(), Vg_all[u][:, :n].cpu().numpy()
            if self.wl.kv_dtype == B.SC_KV_I4G64:
                Km, Vm = self.cache.kv_meta()
                Kg = dequant_i4(Kg, Km[u][:, :n].cpu().numpy())
                Vg = dequant_i4(Vg, Vm[u][:, :n].cpu().numpy())
            Kr, Vr = seq.rows()
            assert np.array_equal(Kg.astype(np.float32), Kr), "sequence %d: stored K rows differ" % b
            assert np.array_equal(Vg.astype(np.float32), Vr), "sequence %d: stored V rows differ" % b

    def run(self):
        for s in range(self.steps_total):
            if self.step(s):
                self.compress()
        self.check_state()
        return self.stats
