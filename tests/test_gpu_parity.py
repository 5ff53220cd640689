"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle.

Small shapes first (every storage type and head size, both trigger policies, both threshold
modes, ragged row counts that do not fill a load tile, one to four counter buckets), then
API-level behaviour (prefill == stepping, error codes leave the state untouched).
The five full-size workloads are in test_gpu_workloads.py.
"""
import numpy as np
import pytest
import torch

from paper_2305_17118_amd import binding as B
from paper_2305_17118_amd.workloads import KV_F16, KV_F32, KV_I4G64, Workload, streams

from oracle.sco import Oracle, OracleConfig

from .parity_util import ParityRun

pytestmark = pytest.mark.gpu


def _wl(name, batch, heads, d, kv, prompt, decode, budget, r, w, m, heavy=0.0, cid=90):
    return Workload(name, cid, batch, heads, d, kv, prompt, decode, budget, r, w, m, heavy)


SMALL = [
    # name, batch, heads, d, kv, prompt, decode, B, r, w, m, heavy
    _wl("f32-d64", 1, 3, 64, KV_F32, 100, 60, 40, 5, 16, 8),
    _wl("f32-d128", 1, 2, 128, KV_F32, 90, 30, 37, 3, 12, 6),
    _wl("f16-d128-ragged", 1, 5, 128, KV_F16, 150, 100, 100, 7, 32, 16, 0.05),
    _wl("f16-d64", 2, 2, 64, KV_F16, 120, 40, 50, 4, 20, 10),
    _wl("i4-d128", 1, 4, 128, KV_I4G64, 130, 60, 70, 6, 24, 12, 0.05),
    _wl("i4-d64", 1, 3, 64, KV_I4G64, 100, 40, 45, 4, 16, 8),
    _wl("drop-one", 1, 2, 128, KV_F16, 60, 40, 30, 1, 4, 1),
    _wl("one-bucket", 1, 2, 64, KV_F32, 80, 40, 33, 2, 9, 9),
    _wl("four-buckets", 1, 3, 128, KV_F16, 120, 80, 64, 8, 32, 8, 0.1),
    _wl("long-window", 1, 2, 128, KV_F16, 90, 60, 20, 2, 64, 8),  # w > trigger size
]


@pytest.mark.parametrize("wl", SMALL, ids=lambda w: w.name)
@pytest.mark.parametrize("trigger", [B.SC_TRIGGER_HARD_CAP, B.SC_TRIGGER_HIGH_WATER], ids=["cap", "hw"])
def test_small_shapes_match_oracle(wl, trigger):
    run = ParityRun(wl, trigger=trigger)
    st = run.run()
    assert st["steps"] == wl.total and st["compressions"] >= 3
    n_after = wl.budget + 1 - wl.drop if trigger == B.SC_TRIGGER_HARD_CAP else wl.budget
    assert run.cache.n_trig - wl.drop == n_after


@pytest.mark.parametrize("kv,d", [(KV_F32, 64), (KV_F16, 128), (KV_I4G64, 128)])
def test_threshold_on_resident_count_and_explicit_scale(kv, d):
    wl = _wl("inv-len", 1, 3, d, kv, 80, 50, 36, 4, 16, 8, 0.05)
    st = ParityRun(wl, thresh=B.SC_THRESH_INV_LEN, scale=0.11).run()
    assert st["compressions"] >= 5


@pytest.mark.parametrize("units,kv", [(1100, KV_F16), (2100, KV_F16), (520, KV_I4G64), (1030, KV_I4G64),
                                      (2060, KV_I4G64), (2050, KV_F32)])
def test_many_units_select_other_workgroup_shapes(units, kv):
    """Unit counts on both sides of the points where the launcher changes the workgroup size."""
    d = 64 if kv == KV_F32 else 128
    wl = _wl("units-%d" % units, units // 10, 10, d, kv, 70, 30, 48, 5, 16, 16, 0.05)
    sel = [0, 1, 63, 64, wl.units // 2, wl.units - 2, wl.units - 1]
    st = ParityRun(wl, sel=sel).run()
    assert st["compressions"] >= 3


@pytest.mark.parametrize("kv,d", [(KV_F16, 128), (KV_I4G64, 128), (KV_F32, 64)])
def test_extreme_window_parameters(kv, d):
    """Degenerate settings: every row outside the recent window is dropped at each compression
    (m = n_trig - r), and a recent window that leaves exactly m candidates."""
    wl = _wl("drop-all-candidates", 1, 3, d, kv, 60, 40, 24, 5, 20, 20)   # n_trig 25, m = 25 - 5
    run = ParityRun(wl)
    st = run.run()
    assert st["compressions"] >= 4 and run.cache.n <= 24
    wl = _wl("recent-is-almost-everything", 1, 2, d, kv, 50, 30, 24, 21, 8, 4)  # candidates = m = 4
    st = ParityRun(wl).run()
    assert st["compressions"] >= 10


def test_maximum_capacity():
    """The largest cache the library accepts (12288 slots: one unit's scores fill the LDS budget),
    driven to its first compression and beyond; every 64th step and the steps around the
    compression are compared with the oracle, all integer state bit for bit."""
    cap = 12288
    wl = _wl("max-capacity", 1, 2, 128, KV_F16, cap, 40, cap - 1, 64, 512, 256, 0.02)
    run = ParityRun(wl)
    for s in range(wl.total):
        near = abs(s + 1 - cap) <= 2
        due = run.step(check=(s % 64 == 0) or near or s == wl.total - 1)
        if due:
            run.compress(check_rows=True)
    assert run.stats["compressions"] == 1 and run.cache.n == cap - 256 + 40
    cfg = B.make_config(1, 2, 128, KV_F16, cap, 64, 512, 256)
    with pytest.raises(B.ScError) as e:
        B.sc_config_sizes(cfg)  # n_trig = 12289 does not fit
    assert e.value.status == B.SC_ERR_UNSUPPORTED


@pytest.mark.parametrize("kv,d", [(KV_F16, 128), (KV_I4G64, 128), (KV_F32, 64), (KV_I4G64, 64)])
@pytest.mark.parametrize("B_,r,w,m", [(40, 3, 7, 5), (64, 10, 40, 32), (50, 4, 33, 8), (30, 2, 70, 9)])
def test_exact_ring_window_for_any_history_length(kv, d, B_, r, w, m):
    """History windows that are not a multiple of the drop amount use the exact ring (one bit
    per row and step); records must equal the oracle's sliding window bit for bit."""
    wl = _wl("ring-w%d-m%d" % (w, m), 1, 3, d, kv, 3 * B_, B_, B_, r, w, m, 0.05)
    run = ParityRun(wl)
    assert run.cache.ring_words == (w + 31) // 32 and run.cache.buckets == 0
    st = run.run()
    assert st["compressions"] >= 6


def test_ring_and_buckets_agree_where_both_apply():
    """Forcing the ring on a window that buckets also cover gives the same evictions."""
    wl = _wl("ring-forced", 1, 4, 128, KV_F16, 150, 80, 64, 8, 32, 16, 0.1)
    a = ParityRun(wl)
    b = ParityRun(wl, window_mode=B.SC_WINDOW_RING)
    assert a.cache.buckets == 2 and b.cache.ring_words == 1
    sa, sb = a.run(), b.run()
    assert sa["compressions"] == sb["compressions"] >= 10
    assert np.array_equal(a.oracle.positions(), b.oracle.positions())


def test_papers_hyper_parameters():
    """r = 10, w = 400, m = B/2 (Sec. 4.1 and the "Overhead Tradeoff" paragraph) on an
    OPT-6.7B-shaped head count, 2x compression of a 1024-token stream."""
    wl = _wl("paper-r10-w400-mhalf", 2, 32, 128, KV_F16, 768, 256, 512, 10, 400, 256, 0.05)
    run = ParityRun(wl, sel=[0, 1, 31, 32, 63])
    assert run.cache.ring_words == 13
    st = run.run(check_rows_every=2)
    assert st["compressions"] == 2 + 0 * wl.total and run.cache.n <= 513


def test_budget_not_reached_is_full_attention():
    wl = _wl("no-evict", 1, 4, 128, KV_F16, 40, 30, 128, 8, 32, 16)
    run = ParityRun(wl)
    st = run.run()
    assert st["compressions"] == 0 and run.cache.n == 70
    # textbook attention over everything seen so far, straight from the inputs
    q, k, v = (a.astype(np.float64) for a in streams(wl))
    lg = np.einsum("ud,utd->ut", q[:, -1], k) / np.sqrt(128)
    p = np.exp(lg - lg.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    ref = np.einsum("ut,utd->ud", p, v)
    got = run.out.float().cpu().numpy()
    assert np.all(np.linalg.norm(got - ref, axis=1) <= 2e-3 * np.linalg.norm(ref, axis=1))


def test_streamed_prefill_equals_stepping():
    """sc_prefill (streamed mode) is the prompt streamed through decode steps with a compression whenever one
    is due: cache contents, counters, positions and outputs must be identical, bit for bit."""
    wl = _wl("prefill", 2, 3, 128, KV_F16, 200, 0, 64, 8, 32, 16, 0.05)
    q, k, v = (torch.from_numpy(a).cuda() for a in streams(wl))
    cfg = B.make_config(wl.batch, wl.heads, wl.head_dim, wl.kv_dtype, wl.budget, wl.recent, wl.history,
                        wl.drop)
    a, b = B.BudgetCache(cfg), B.BudgetCache(cfg)
    T, d, U = wl.total, wl.head_dim, wl.units
    out_a = torch.empty(U, T, d, dtype=torch.float16, device="cuda")
    out_b = torch.zeros(U, T, d, dtype=torch.float16, device="cuda")
    a.prefill(q, k, v, T, 0, out_a, mode=B.SC_PREFILL_STREAMED)
    step_out = torch.empty(U, d, dtype=torch.float16, device="cuda")
    for s in range(T):
        due = b.decode_step(q[:, s], k[:, s], v[:, s], step_out, in_stride=T * d)
        out_b[:, s] = step_out
        if due:
            b.compress()
    assert (a.n, a.t) == (b.n, b.t)
    n = a.n
    assert torch.equal(out_a, out_b)
    assert torch.equal(a.pos()[:, :n], b.pos()[:, :n])
    assert torch.equal(a.cnt(), b.cnt())
    Ka, Va = a.kv_rows()
    Kb, Vb = b.kv_rows()
    assert torch.equal(Ka[:, :n], Kb[:, :n]) and torch.equal(Va[:, :n], Vb[:, :n])
    # a strided prompt (longer allocation than the prompt) gives the same cache
    c = B.BudgetCache(cfg)
    pad = torch.zeros(U, 8, d, dtype=torch.float16, device="cuda")
    qq, kk, vv = (torch.cat([x, pad], dim=1).contiguous() for x in (q, k, v))
    c.prefill(qq, kk, vv, T, (T + 8) * d, None, mode=B.SC_PREFILL_STREAMED)
    assert torch.equal(a.pos()[:, :n], c.pos()[:, :n]) and torch.equal(a.cnt(), c.cnt())


DENSE_PREFILL = [
    # name, batch, heads, d, kv, prompt, decode, B, r, w, m, heavy
    _wl("pf-d128", 1, 4, 128, KV_F16, 400, 70, 150, 8, 96, 48, 0.05),       # runs of 48 and a first run of 151
    _wl("pf-d64", 2, 2, 64, KV_F16, 333, 50, 100, 6, 64, 32, 0.05),
    _wl("pf-short-prompt", 1, 3, 128, KV_F16, 37, 200, 90, 5, 60, 30),      # prompt ends before the first boundary
    _wl("pf-long-runs", 1, 2, 128, KV_F16, 700, 150, 300, 16, 400, 200, 0.03),  # runs of 200 = 4 query blocks
    _wl("pf-tiny-drop", 1, 2, 64, KV_F16, 150, 40, 60, 4, 16, 4),           # runs of 4: streamed inside AUTO
    _wl("pf-mixed", 1, 3, 128, KV_F16, 260, 60, 77, 7, 51, 17, 0.1),        # runs of 17: one ragged query block
    _wl("pf-i4", 1, 4, 128, KV_I4G64, 400, 70, 150, 8, 96, 48, 0.05),       # 4-bit rows quantised by the run
    _wl("pf-i4-long-runs", 2, 2, 128, KV_I4G64, 700, 120, 300, 16, 400, 200, 0.03),
    _wl("pf-i4-ragged", 1, 3, 128, KV_I4G64, 260, 60, 77, 7, 51, 17, 0.1),
    _wl("pf-i4-d64", 1, 2, 64, KV_I4G64, 150, 40, 60, 4, 32, 16),           # 4-bit rows of one 64-channel group
    _wl("pf-i4-d64-long-runs", 2, 3, 64, KV_I4G64, 700, 120, 300, 16, 400, 200, 0.03),
    _wl("pf-f32-d64", 1, 2, 64, KV_F32, 150, 40, 60, 4, 32, 16),            # fp32 rows on the fp32 matrix instruction
    _wl("pf-f32-d128", 2, 2, 128, KV_F32, 400, 70, 150, 8, 96, 48, 0.05),
    _wl("pf-f32-long-runs", 1, 3, 64, KV_F32, 700, 120, 300, 16, 400, 200, 0.03),
    _wl("pf-f32-ragged", 1, 3, 128, KV_F32, 260, 60, 77, 7, 51, 17, 0.1),
]


@pytest.mark.parametrize("wl", DENSE_PREFILL, ids=lambda w: w.name)
@pytest.mark.parametrize("trigger", [B.SC_TRIGGER_HARD_CAP, B.SC_TRIGGER_HIGH_WATER], ids=["cap", "hw"])
def test_dense_prefill_matches_oracle(wl, trigger):
    """The prompt goes through one sc_prefill call (dense causal blocks on the matrix cores);
    every position is compared with the oracle, then decoding continues so that the
    compressions that follow check the records accumulated during the prompt bit for bit."""
    run = ParityRun(wl, trigger=trigger)
    run.prefill(wl.prompt)
    st = run.run()
    assert st["steps"] == wl.total and st["compressions"] >= 2


RING_PREFILL = [
    # name, batch, heads, d, kv, prompt, decode, B, r, w, m, heavy  (w no multiple of m: ring record)
    _wl("pf-ring-d128", 1, 4, 128, KV_F16, 400, 70, 150, 8, 100, 48, 0.05),
    _wl("pf-ring-d64", 2, 2, 64, KV_F16, 333, 50, 100, 6, 45, 32, 0.05),
    _wl("pf-ring-paper", 1, 3, 128, KV_F16, 700, 300, 400, 10, 400, 200, 0.05),   # r = 10, w = 400, m = B/2
    _wl("pf-ring-short-window", 1, 2, 128, KV_F16, 300, 60, 100, 8, 5, 48),        # w far below a query block
    _wl("pf-ring-window-33", 1, 3, 128, KV_F16, 350, 80, 120, 8, 33, 64, 0.1),    # w < run length, odd word split
    _wl("pf-ring-long-window", 1, 2, 64, KV_F16, 260, 90, 77, 7, 1000, 17, 0.1),  # w beyond everything seen
    _wl("pf-ring-i4", 1, 4, 128, KV_I4G64, 400, 70, 150, 8, 100, 48, 0.05),        # 4-bit rows, ring record
    _wl("pf-ring-i4-paper", 1, 2, 128, KV_I4G64, 700, 300, 400, 10, 400, 200, 0.05),
    _wl("pf-ring-i4-window-33", 2, 2, 128, KV_I4G64, 350, 80, 120, 8, 33, 64, 0.1),
    _wl("pf-ring-i4-d64", 2, 2, 64, KV_I4G64, 333, 50, 100, 6, 45, 32, 0.05),
    _wl("pf-ring-f32", 2, 2, 64, KV_F32, 333, 50, 100, 6, 45, 32, 0.05),
    _wl("pf-ring-f32-d128", 1, 2, 128, KV_F32, 350, 80, 120, 8, 33, 64, 0.1),
]


@pytest.mark.parametrize("wl", RING_PREFILL, ids=lambda w: w.name)
def test_dense_prefill_with_ring_record_matches_oracle(wl):
    """Dense prompt runs writing the one-bit-per-step record: every position compared, then the
    decode steps' compressions check the rings the prompt left behind bit for bit."""
    run = ParityRun(wl, window_mode=B.SC_WINDOW_RING)
    assert any(dense for _, dense, _ in B.sc_prefill_plan(run.cfg, wl.prompt))
    run.prefill(wl.prompt)
    st = run.run()
    assert st["steps"] == wl.total and st["compressions"] >= 2


@pytest.mark.parametrize("kv,window", [(KV_F16, B.SC_WINDOW_AUTO), (KV_I4G64, B.SC_WINDOW_AUTO),
                                       (KV_F16, B.SC_WINDOW_RING), (KV_F32, B.SC_WINDOW_AUTO)],
                         ids=["f16", "i4", "f16-ring", "f32"])
def test_prefill_continues_a_cache_that_is_not_empty(kv, window):
    """A prompt handed over in chunks, decode steps, then a later turn's prompt: every sc_prefill
    call continues the stream from wherever the cache stands (chunks that start in the middle of
    a run between two compressions, right after a compression, and after decode steps)."""
    d = 64 if kv == KV_F32 else 128
    wl = _wl("pf-chunks", 1, 3, d, kv, 0, 700, 150, 8, 96, 48, 0.05)
    run = ParityRun(wl, window_mode=window)
    run.prefill(100)        # ends before the first compression
    run.prefill(51)         # reaches the trigger size exactly: the compression happens inside
    assert run.cache.n == 151 - 48
    run.prefill(130)        # several runs, starts right after a compression
    run.run(steps=75)       # decode steps (with their own compressions)
    run.prefill(200)        # a later turn: starts in the middle of a run
    run.prefill(1)          # a single position
    st = run.run()
    assert st["steps"] == wl.total and st["compressions"] >= 8


def test_dense_prefill_inverse_length_threshold():
    wl = _wl("pf-inv-len", 1, 3, 128, KV_F16, 300, 80, 120, 8, 64, 32, 0.05)
    run = ParityRun(wl, thresh=B.SC_THRESH_INV_LEN, scale=0.2)
    run.prefill(wl.prompt)
    run.run()


def test_dense_and_streamed_prefill_agree():
    """Both modes compute the same function; with well separated scores they evict the same
    rows, and their outputs differ by rounding only."""
    wl = _wl("pf-modes", 1, 4, 128, KV_F16, 300, 0, 100, 8, 64, 32, 0.05)
    q, k, v = (torch.from_numpy(a).cuda() for a in streams(wl))
    cfg = B.make_config(wl.batch, wl.heads, wl.head_dim, wl.kv_dtype, wl.budget, wl.recent, wl.history,
                        wl.drop)
    a, b = B.BudgetCache(cfg), B.BudgetCache(cfg)
    T, d, U = wl.total, wl.head_dim, wl.units
    out_a = torch.empty(U, T, d, dtype=torch.float16, device="cuda")
    out_b = torch.empty(U, T, d, dtype=torch.float16, device="cuda")
    a.prefill(q, k, v, T, 0, out_a, mode=B.SC_PREFILL_AUTO)
    b.prefill(q, k, v, T, 0, out_b, mode=B.SC_PREFILL_STREAMED)
    assert (a.n, a.t) == (b.n, b.t) and not torch.equal(out_a, out_b)  # two different computations
    same = (a.pos()[:, :a.n] == b.pos()[:, :b.n]).float().mean().item()
    assert same > 0.9  # a probability within rounding of its threshold may flip one eviction
    err = (out_a.float() - out_b.float()).norm(dim=-1) / out_b.float().norm(dim=-1)
    assert err.median().item() < 2e-3


RECOMPUTE = [
    # name, batch, heads, d, kv, prompt, decode, B, r, w, m, heavy
    _wl("re-d128", 1, 4, 128, KV_F16, 150, 100, 100, 7, 32, 16, 0.05),
    _wl("re-d64", 2, 2, 64, KV_F16, 120, 60, 50, 4, 20, 10),
    _wl("re-paper-params", 1, 3, 128, KV_F16, 300, 400, 200, 10, 400, 100, 0.05),  # w = 400: 7 query blocks
    _wl("re-window-longer-than-cache", 1, 2, 128, KV_F16, 90, 80, 20, 2, 64, 8),   # old steps see few rows
    _wl("re-drop-one", 1, 2, 64, KV_F16, 40, 30, 24, 1, 5, 1),
    _wl("re-i4", 1, 4, 128, KV_I4G64, 150, 100, 100, 7, 32, 16, 0.05),             # 4-bit rows replayed from their codes
    _wl("re-i4-paper-params", 1, 2, 128, KV_I4G64, 300, 400, 200, 10, 400, 100, 0.05),
    _wl("re-i4-window-longer-than-cache", 2, 2, 128, KV_I4G64, 90, 80, 20, 2, 64, 8),
    _wl("re-i4-d64", 2, 3, 64, KV_I4G64, 120, 90, 50, 4, 70, 10, 0.05),
    _wl("re-f32-d64", 2, 2, 64, KV_F32, 120, 60, 50, 4, 20, 10),
    _wl("re-f32-d128", 1, 3, 128, KV_F32, 150, 100, 100, 7, 32, 16, 0.05),
]


@pytest.mark.parametrize("wl", RECOMPUTE, ids=lambda w: w.name)
@pytest.mark.parametrize("thresh", [B.SC_THRESH_INV_POS, B.SC_THRESH_INV_LEN], ids=["inv-t", "inv-n"])
def test_recomputed_record_matches_oracle(wl, thresh):
    """Alg. 2 as printed: no counting during the steps; at every compression the last w
    queries are replayed over the resident rows.  Steps are compared as always; at each
    compression the replayed probabilities are compared and the evicted slots must agree."""
    run = ParityRun(wl, thresh=thresh, record_mode=B.SC_RECORD_RECOMPUTE)
    st = run.run()
    assert st["steps"] == wl.total and st["compressions"] >= 3


@pytest.mark.parametrize("kv", [KV_F16, KV_I4G64, KV_F32], ids=["f16", "i4", "f32"])
def test_recomputed_record_after_dense_prefill(kv):
    """The queries of a prompt that went through sc_prefill are kept too: the compressions
    during the decode steps that follow replay them."""
    wl = _wl("re-prefill", 1, 4, 128, kv, 90, 120, 100, 8, 64, 32, 0.05)  # prompt ends before the trigger
    run = ParityRun(wl, record_mode=B.SC_RECORD_RECOMPUTE)
    run.prefill(wl.prompt)
    st = run.run()
    assert st["compressions"] >= 3


@pytest.mark.parametrize("kv,d,window,record", [
    (KV_F16, 128, B.SC_WINDOW_AUTO, B.SC_RECORD_ONLINE), (KV_F32, 64, B.SC_WINDOW_AUTO, B.SC_RECORD_ONLINE),
    (KV_I4G64, 128, B.SC_WINDOW_AUTO, B.SC_RECORD_ONLINE), (KV_I4G64, 64, B.SC_WINDOW_AUTO, B.SC_RECORD_ONLINE),
    (KV_F16, 128, B.SC_WINDOW_RING, B.SC_RECORD_ONLINE), (KV_F16, 128, B.SC_WINDOW_AUTO, B.SC_RECORD_RECOMPUTE),
    (KV_I4G64, 128, B.SC_WINDOW_AUTO, B.SC_RECORD_RECOMPUTE)],
    ids=["f16", "f32", "i4-d128", "i4-d64", "f16-ring", "f16-recompute", "i4-recompute"])
def test_decode_without_dumps_leaves_the_same_state(kv, d, window, record):
    """The benchmark's path: no `probs_out`, no `evicted_out`.  Outputs, records, positions and
    stored rows must be exactly those of the instrumented calls the parity tests compare."""
    wl = _wl("prod", 2, 3, d, kv, 0, 150, 64, 8, 32, 16, 0.05)
    T, U = wl.total, wl.units
    q, k, v = (torch.from_numpy(a).cuda() for a in streams(wl))
    cfg = B.make_config(wl.batch, wl.heads, d, kv, wl.budget, wl.recent, wl.history, wl.drop,
                        window_mode=window, record_mode=record)
    a, b = B.BudgetCache(cfg), B.BudgetCache(cfg)
    out_a = torch.empty(U, d, dtype=a.io_dtype, device="cuda")
    out_b = torch.empty_like(out_a)
    probs = torch.zeros(U, a.capacity, dtype=torch.float32, device="cuda")
    ev = torch.empty(U, wl.drop, dtype=torch.int32, device="cuda")
    re_probs = torch.zeros(U, wl.history, a.capacity, dtype=torch.float32, device="cuda")
    compressions = 0
    for s in range(T):
        due_a = a.decode_step(q[:, s], k[:, s], v[:, s], out_a, probs, in_stride=T * d)
        due_b = b.decode_step(q[:, s], k[:, s], v[:, s], out_b, None, in_stride=T * d)
        assert due_a == due_b and torch.equal(out_a, out_b), "step %d" % s
        if due_a:
            a.compress(ev, re_probs if record == B.SC_RECORD_RECOMPUTE else None)
            b.compress()
            compressions += 1
    assert compressions >= 5 and (a.n, a.t) == (b.n, b.t)
    n = a.n
    planes_a, planes_b = (c.ring() if c.ring_words else c.cnt() for c in (a, b))
    assert torch.equal(planes_a, planes_b) and torch.equal(a.pos()[:, :n], b.pos()[:, :n])
    for xa, xb in zip(a.kv_rows(), b.kv_rows()):
        assert torch.equal(xa[:, :n], xb[:, :n])


@pytest.mark.parametrize("kv", [KV_F16, KV_I4G64], ids=["f16", "i4"])
def test_dense_prefill_production_path_and_reset(kv):
    """The dumps are optional: a call without `out` and `probs_out` (the second pass then only
    counts), a call on strided inputs, and a call on a cache that was used and reset must all
    leave exactly the state of the fully instrumented call."""
    wl = _wl("pf-prod", 2, 3, 128, kv, 300, 0, 100, 8, 64, 32, 0.05)
    T, d, U = wl.total, wl.head_dim, wl.units
    q, k, v = (torch.from_numpy(a).cuda() for a in streams(wl))
    cfg = B.make_config(wl.batch, wl.heads, wl.head_dim, wl.kv_dtype, wl.budget, wl.recent, wl.history,
                        wl.drop)

    def state(c):
        n = c.n
        K, V = c.kv_rows()
        out = [c.pos()[:, :n].clone(), c.cnt().clone(), K[:, :n].clone(), V[:, :n].clone()]
        if kv == KV_I4G64:
            Km, Vm = c.kv_meta()
            out += [Km[:, :n].clone(), Vm[:, :n].clone()]
        return (n, c.t), out

    full = B.BudgetCache(cfg)
    out = torch.empty(U, T, d, dtype=torch.float16, device="cuda")
    probs = torch.zeros(U, T, full.capacity, dtype=torch.float32, device="cuda")
    full.prefill(q, k, v, T, 0, out, probs)
    ref = state(full)

    def same(c):
        got = state(c)
        return got[0] == ref[0] and all(torch.equal(a, b) for a, b in zip(got[1], ref[1]))

    bare = B.BudgetCache(cfg)
    bare.prefill(q, k, v, T)
    assert same(bare)
    pad = torch.zeros(U, 8, d, dtype=torch.float16, device="cuda")
    qq, kk, vv = (torch.cat([x, pad], dim=1).contiguous() for x in (q, k, v))
    strided = B.BudgetCache(cfg)
    out2 = torch.empty_like(out)
    strided.prefill(qq, kk, vv, T, (T + 8) * d, out2)
    assert same(strided) and torch.equal(out2, out)
    # a used cache, reset: counters, lengths and schedule start over
    bare.reset()
    assert (bare.n, bare.t) == (0, 0)
    bare.prefill(q, k, v, T, 0, out2)
    assert same(bare) and torch.equal(out2, out)
    with pytest.raises(B.ScError) as e:
        B.BudgetCache(cfg).prefill(q, k, v, T, mode=5)
    assert e.value.status == B.SC_ERR_INVALID_ARG


def test_error_codes_leave_state_untouched():
    wl = _wl("errors", 1, 2, 64, KV_F32, 0, 0, 8, 2, 4, 4)
    cfg = B.make_config(1, 2, 64, KV_F32, 8, 2, 4, 4)
    c = B.BudgetCache(cfg)
    x = torch.randn(2, 64, device="cuda")
    out = torch.empty(2, 64, device="cuda")
    with pytest.raises(B.ScError) as e:
        c.compress()
    assert e.value.status == B.SC_ERR_STATE
    for i in range(9):
        due = c.decode_step(x, x, x, out)
        assert due == (i == 8)
    assert (c.n, c.t) == (9, 9)
    with pytest.raises(B.ScError) as e:
        c.decode_step(x, x, x, out)
    assert e.value.status == B.SC_ERR_FULL and (c.n, c.t) == (9, 9)
    with pytest.raises(B.ScError) as e:
        c.prefill(x, x, x, 1)  # a compression is due
    assert e.value.status == B.SC_ERR_FULL and (c.n, c.t) == (9, 9)
    with pytest.raises(B.ScError) as e:
        B.sc_decode_step(c.handle, x.data_ptr() + 4, x.data_ptr(), x.data_ptr(), 0, out.data_ptr())
    assert e.value.status == B.SC_ERR_INVALID_ARG
    c.compress()
    assert (c.n, c.t) == (5, 9)
    with pytest.raises(B.ScError) as e:
        B.sc_decode_step(c.handle, None, x.data_ptr(), x.data_ptr(), 0, out.data_ptr())
    assert e.value.status == B.SC_ERR_INVALID_ARG and (c.n, c.t) == (5, 9)
    probs = torch.zeros(2, c.capacity + 2, device="cuda")
    with pytest.raises(B.ScError) as e:  # probabilities are stored in pairs: 8-byte alignment
        B.sc_decode_step(c.handle, x.data_ptr(), x.data_ptr(), x.data_ptr(), 0, out.data_ptr(),
                         probs.data_ptr() + 4)
    assert e.value.status == B.SC_ERR_INVALID_ARG and (c.n, c.t) == (5, 9)
    with pytest.raises(B.ScError) as e:
        B.sc_decode_step_ragged(c.handle, x.data_ptr(), x.data_ptr(), x.data_ptr(), 0, out.data_ptr(),
                                probs.data_ptr() + 4)
    assert e.value.status == B.SC_ERR_INVALID_ARG and (c.n, c.t) == (5, 9)  # still a lock-step handle
    fresh = B.BudgetCache(cfg)
    with pytest.raises(B.ScError) as e:
        fresh.prefill(x, x, x, 0)
    assert e.value.status == B.SC_ERR_INVALID_ARG
    torch.cuda.synchronize()


@pytest.mark.parametrize("kv", [KV_F16, KV_I4G64, KV_F32], ids=["f16", "i4", "f32"])
def test_free_running_oracle_divergence_is_reported(kv, record_property):
    """Without forcing: the oracle decides low scores from its own double-precision
    probabilities, the GPU from its fp32 ones.  A probability within rounding of its threshold
    can then flip a flag, and a flipped flag can change an eviction, after which the two caches
    hold different rows.  Not gated on equality: the agreement is measured and reported (final
    resident positions in common, units whose whole history agrees); it only has to be high."""
    d = 64 if kv == KV_F32 else 128
    wl = _wl("free", 2, 4, d, kv, 0, 420, 96, 8, 64, 32, 0.05)
    T, U = wl.total, wl.units
    q, k, v = streams(wl, steps=T)
    tq, tk, tv = (torch.from_numpy(a).cuda() for a in (q, k, v))
    cfg = B.make_config(wl.batch, wl.heads, d, kv, wl.budget, wl.recent, wl.history, wl.drop)
    cache = B.BudgetCache(cfg)
    oracle = Oracle(OracleConfig(wl.batch, wl.heads, d, kv, wl.budget, wl.recent, wl.history, wl.drop))
    out = torch.empty(U, d, dtype=cache.io_dtype, device="cuda")
    ev = torch.empty(U, wl.drop, dtype=torch.int32, device="cuda")
    agree = np.ones(U, dtype=bool)  # units whose evictions have all agreed so far
    comps = same_lists = 0
    for s in range(T):
        due = cache.decode_step(tq[:, s], tk[:, s], tv[:, s], out, in_stride=T * d)
        _, _, due_ref = oracle.step(q[:, s], k[:, s], v[:, s], want_probs=False)
        assert due == due_ref
        if due:
            cache.compress(ev)
            ev_ref = oracle.compress()
            same = (ev.cpu().numpy() == ev_ref).all(axis=1)
            same_lists += int((same & agree).sum())
            comps += int(agree.sum())
            agree &= same
    n = cache.n
    pos_gpu = cache.pos()[:, :n].cpu().numpy()
    pos_ref = oracle.positions()
    common = np.mean([len(np.intersect1d(pos_gpu[u], pos_ref[u])) / n for u in range(U)])
    record_property("units_with_identical_history", float(agree.mean()))
    record_property("resident_positions_in_common", float(common))
    print("\nfree-running %s: %d/%d units keep identical evictions over %d compressions each; "
          "%.4f of the final resident positions in common" % (
              ("f32", "f16", "i4")[kv], int(agree.sum()), U, comps // max(1, U), common), flush=True)
    assert common >= 0.9


PATTERNS = ["random", "front", "back", "alternate", "block", "two-blocks"]


@pytest.mark.parametrize("pattern", PATTERNS)
@pytest.mark.parametrize("kv,d", [(KV_F16, 128), (KV_I4G64, 128), (KV_F32, 64), (KV_F16, 64)],
                         ids=["f16", "i4", "f32", "f16-d64"])
def test_in_place_compaction_equals_out_of_place_gather(kv, d, pattern):
    """The compaction moves rows inside the arrays it reads.  Here the records are written by the
    test so that Alg. 2 must evict a chosen set of slots (each unit its own), and the result is
    compared with an out-of-place gather of the snapshot taken before: stored rows, 4-bit
    meta words, positions and the surviving counter bucket, for eviction patterns that stress the
    chunked in-place move (evictions at the very front, right below the recent window,
    alternating, in blocks)."""
    m, r, budget = 96, 8, 299  # trigger size 300, not a multiple of the 64-slot capacity rounding
    wl = _wl("compact", 2, 3, d, kv, 0, budget + 1, budget, r, 2 * m, m)
    U, n = wl.units, budget + 1
    q, k, v = (torch.from_numpy(a).cuda() for a in streams(wl))
    cfg = B.make_config(wl.batch, wl.heads, d, kv, budget, r, 2 * m, m)
    cache = B.BudgetCache(cfg)
    out = torch.empty(U, d, dtype=cache.io_dtype, device="cuda")
    due = False
    for s in range(n):
        due = cache.decode_step(q[:, s], k[:, s], v[:, s], out, in_stride=n * d)
    assert due and cache.n == n
    rng = np.random.default_rng(1000 * kv + d + 7919 * PATTERNS.index(pattern))
    ncand = n - r
    chosen = np.zeros((U, m), dtype=np.int64)
    for u in range(U):
        if pattern == "random":
            c = rng.choice(ncand, m, replace=False)
        elif pattern == "front":
            c = np.arange(m)
        elif pattern == "back":
            c = np.arange(ncand - m, ncand)
        elif pattern == "alternate":
            c = np.arange(u % 2, u % 2 + 2 * m, 2)
        elif pattern == "block":
            start = int(rng.integers(0, ncand - m + 1))
            c = np.arange(start, start + m)
        else:
            a = int(rng.integers(0, 60))
            b_ = int(rng.integers(a + m // 2 + 1, ncand - m // 2 + 1))
            c = np.concatenate([np.arange(a, a + m // 2), np.arange(b_, b_ + m // 2)])
        chosen[u] = np.sort(c)
    cnt = cache.cnt()  # [U, 2, C] view into the workspace
    marks = torch.zeros(U, cache.capacity, dtype=torch.int16, device="cuda")
    marks.scatter_(1, torch.from_numpy(chosen).cuda(), 7)
    t = cache.t
    live = 1 - B.sc_schedule(cfg, t + 1)[1]  # the bucket the next epoch does NOT reuse survives
    cnt.zero_()
    cnt[:, live] = marks
    K0, V0 = (x.clone() for x in cache.kv_rows())
    pos0 = cache.pos().clone()
    meta0 = [x.clone() for x in cache.kv_meta()] if kv == KV_I4G64 else None
    ev = torch.empty(U, m, dtype=torch.int32, device="cuda")
    cache.compress(ev)
    assert np.array_equal(ev.cpu().numpy(), chosen)
    keep = np.stack([np.setdiff1d(np.arange(n), chosen[u]) for u in range(U)])
    kt = torch.from_numpy(keep).cuda()
    nn = n - m
    assert cache.n == nn

    def gathered(x):
        idx = kt.view(U, nn, *([1] * (x.dim() - 2))).expand(U, nn, *x.shape[2:])
        return torch.gather(x[:, :n], 1, idx)

    K1, V1 = cache.kv_rows()
    assert torch.equal(K1[:, :nn], gathered(K0)) and torch.equal(V1[:, :nn], gathered(V0))
    assert torch.equal(cache.pos()[:, :nn], gathered(pos0))
    if meta0 is not None:
        Km1, Vm1 = cache.kv_meta()
        assert torch.equal(Km1[:, :nn], gathered(meta0[0])) and torch.equal(Vm1[:, :nn], gathered(meta0[1]))
    c1 = cache.cnt()
    assert int(c1[:, live, :nn].abs().max().item()) == 0  # every marked row is gone
    assert int(c1[:, :, nn:].abs().max().item()) == 0 and int(c1[:, 1 - live].abs().max().item()) == 0


@pytest.mark.parametrize("kv", [KV_F16, KV_I4G64], ids=["f16", "i4"])
def test_prefill_can_be_captured_in_a_graph_and_replayed(kv):
    """The library only enqueues kernels on the caller's stream (no allocation, no memset node,
    no synchronisation), so a reset + prompt pass can be captured in a HIP graph.  The graph is
    replayed several times with eager work and synchronisations in between and the cache's own
    memory scrambled before each replay; every replay must reproduce the eager result bit for bit."""
    wl = _wl("graph", 2, 3, 128, kv, 0, 330, 100, 8, 64, 32, 0.05)
    P, U, d = wl.total, wl.units, wl.head_dim
    q, k, v = (torch.from_numpy(a).cuda() for a in streams(wl))
    cfg = B.make_config(wl.batch, wl.heads, d, kv, wl.budget, wl.recent, wl.history, wl.drop)
    eager = B.BudgetCache(cfg)
    out_e = torch.empty(U, P, d, dtype=torch.float16, device="cuda")
    eager.prefill(q, k, v, P, 0, out_e)
    torch.cuda.synchronize()
    n = eager.n

    def state(c):
        K, V = c.kv_rows()
        return [K[:, :n].clone(), V[:, :n].clone(), c.pos()[:, :n].clone(), c.cnt().clone()]

    want = state(eager)
    cache = B.BudgetCache(cfg)
    out_g = torch.zeros_like(out_e)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        cache.reset()
        cache.prefill(q, k, v, P, 0, out_g)
    assert (cache.n, cache.t) == (eager.n, eager.t)
    other = B.BudgetCache(cfg)  # eager work between the replays
    step_out = torch.empty(U, d, dtype=torch.float16, device="cuda")
    for rep in range(4):
        cache.workspace.random_(0, 255)  # whatever the previous replay left is gone
        out_g.fill_(float("nan"))
        for s in range(5):
            if other.decode_step(q[:, s], k[:, s], v[:, s], step_out, in_stride=P * d):
                other.compress()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e), "replay %d: outputs differ" % rep
        got = state(cache)
        for a, b in zip(got, want):
            assert torch.equal(a, b), "replay %d: cache state differs" % rep


@pytest.mark.parametrize("batch,heads,kv,d,budget", [
    (1, 1, KV_F16, 128, 700),     # a single unit
    (1, 32, KV_F16, 128, 520),    # batch 1 of the headline shape
    (3, 24, KV_F32, 64, 300),
    (2, 80, KV_F16, 64, 290),
    (1, 5, KV_F32, 128, 255),
    (2, 40, KV_F32, 64, 600),
    (1, 3, KV_F16, 64, 513),      # head size 64, capacity just above 512 slots
    (2, 24, KV_F16, 128, 540),    # 48 units: four workgroups per unit
    (1, 4, KV_F32, 64, 600),      # fp32 rows, eight workgroups per unit
])
def test_few_units_with_many_rows(batch, heads, kv, d, budget):
    """Small batches with long caches (the shape of low-latency serving): a streamed prompt, then
    decode steps and compressions, over row counts that are no multiple of anything."""
    wl = _wl("few-units", batch, heads, d, kv, 0, budget + 150, budget, 9, 70, 35, 0.05)
    run = ParityRun(wl)
    run.prefill(budget - 40, mode=B.SC_PREFILL_STREAMED)
    st = run.run()
    assert st["steps"] == wl.total and st["compressions"] >= 4


def test_shared_units_give_the_same_bits_whoever_arrives_last():
    """32 units with long caches: 8 workgroups share a unit's rows and the last of them to arrive
    merges the shares.  Which one that is changes from launch to launch; the result must not:
    two caches fed the same stream, and a third one whose steps are interleaved with unrelated
    work, agree bit for bit on every output and on the final state."""
    wl = _wl("shared-units", 1, 32, 128, KV_F16, 0, 700, 540, 9, 64, 32, 0.05)
    T, U, d = 640, wl.units, wl.head_dim
    q, k, v = (torch.from_numpy(a).cuda() for a in streams(wl, steps=T))
    cfg = B.make_config(wl.batch, wl.heads, d, wl.kv_dtype, wl.budget, wl.recent, wl.history, wl.drop)
    caches = [B.BudgetCache(cfg) for _ in range(3)]
    for c in caches:
        c.prefill(q, k, v, 500, T * d, None)
    outs = [torch.empty(U, d, dtype=torch.float16, device="cuda") for _ in caches]
    noise = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    comps = 0
    for s in range(500, T):
        qs, ks, vs = q[:, s].contiguous(), k[:, s].contiguous(), v[:, s].contiguous()
        due = [c.decode_step(qs, ks, vs, o) for c, o in zip(caches[:2], outs[:2])]
        noise.random_(0, 255)  # other kernels in between shift the third cache's timing
        due.append(caches[2].decode_step(qs, ks, vs, outs[2]))
        assert due[0] == due[1] == due[2]
        assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2]), "step %d" % s
        if due[0]:
            for c in caches:
                c.compress()
            comps += 1
    assert comps >= 3
    n = caches[0].n  # slots beyond the resident rows hold whatever the workspace held
    for c in caches[1:]:
        assert c.n == n and torch.equal(caches[0].cnt(), c.cnt())
        assert torch.equal(caches[0].pos()[:, :n], c.pos()[:, :n])
