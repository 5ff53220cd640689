"""Seeded random configurations: storage type, head size, budget, windows, drop amount, trigger
policy, threshold mode, record layout and record mode, prompt through sc_prefill or through
steps.  Each case is a short run compared with the oracle like every other parity test; the
point is to walk the edges of the tilings (rows resident before a run at any offset inside a
64-row tile, runs shorter and longer than a query block, windows that are no multiple of
anything) without choosing them by hand."""
import numpy as np
import pytest

from paper_2305_17118_amd import binding as B
from paper_2305_17118_amd.workloads import KV_F16, KV_F32, KV_I4G64, Workload

from .parity_util import ParityRun

pytestmark = pytest.mark.gpu


def _draw(seed):
    rng = np.random.default_rng(1000 + seed)
    kv = int(rng.choice([KV_F32, KV_F16, KV_F16, KV_I4G64, KV_I4G64]))
    d = 64 if kv == KV_F32 else int(rng.choice([64, 128]))
    budget = int(rng.integers(20, 260))
    trigger = int(rng.choice([B.SC_TRIGGER_HARD_CAP, B.SC_TRIGGER_HIGH_WATER]))
    m = int(rng.integers(1, max(2, budget // 2)))
    n_trig = budget + 1 if trigger == B.SC_TRIGGER_HARD_CAP else budget + m
    r = int(rng.integers(1, max(2, n_trig - m)))
    record = B.SC_RECORD_ONLINE
    window = B.SC_WINDOW_AUTO
    kind = int(rng.integers(0, 4))
    if kind == 0:      # bucket counters: w a multiple of m
        w = m * int(rng.integers(1, 5))
    elif kind == 1:    # exact ring: any w
        w = int(rng.integers(1, 300))
        window = B.SC_WINDOW_RING
    elif kind == 2 and kv == KV_F16:  # record rebuilt at compression time
        w = int(rng.integers(1, 200))
        record = B.SC_RECORD_RECOMPUTE
    else:
        w = m * int(rng.integers(1, 4))
    w = min(w, 8192)
    thresh = int(rng.choice([B.SC_THRESH_INV_POS, B.SC_THRESH_INV_LEN]))
    prompt = int(rng.integers(1, 2 * n_trig + 3 * m))
    decode = int(rng.integers(m + 2, 3 * m + 40))
    heads = int(rng.integers(1, 5))
    batch = int(rng.integers(1, 3))
    use_prefill = bool(rng.integers(0, 2))
    heavy = float(rng.choice([0.0, 0.05, 0.1]))
    wl = Workload("rnd-%d" % seed, 500 + seed, batch, heads, d, kv, prompt, decode, budget, r, w, m, heavy)
    return wl, trigger, thresh, window, record, use_prefill


@pytest.mark.parametrize("seed", range(40))
def test_random_configuration_matches_oracle(seed):
    wl, trigger, thresh, window, record, use_prefill = _draw(seed)
    print("\n", wl, "trigger", trigger, "thresh", thresh, "window", window, "record", record,
          "prefill" if use_prefill else "stepped", flush=True)
    run = ParityRun(wl, trigger=trigger, thresh=thresh, window_mode=window, record_mode=record)
    n_trig = run.cache.n_trig
    if use_prefill and not (record == B.SC_RECORD_RECOMPUTE and wl.prompt >= n_trig):
        run.prefill(wl.prompt)
    st = run.run()
    assert st["steps"] == wl.total


def _draw_dense(seed):
    """Configurations whose prompt goes through the dense prompt kernels: fp16 (both head sizes)
    or 4-bit rows of 128 channels, bucket counters, runs of at least 16 positions."""
    rng = np.random.default_rng(5000 + seed)
    kv, d = [(KV_F16, 64), (KV_F16, 128), (KV_I4G64, 128)][int(rng.integers(0, 3))]
    m = int(rng.integers(16, 200))
    budget = int(rng.integers(2 * m, 2 * m + 400))
    trigger = int(rng.choice([B.SC_TRIGGER_HARD_CAP, B.SC_TRIGGER_HIGH_WATER]))
    n_trig = budget + 1 if trigger == B.SC_TRIGGER_HARD_CAP else budget + m
    r = int(rng.integers(1, n_trig - m))
    w = m * int(rng.integers(1, 4))
    thresh = int(rng.choice([B.SC_THRESH_INV_POS, B.SC_THRESH_INV_LEN]))
    record = B.SC_RECORD_ONLINE
    prompt = int(rng.integers(2 * m, n_trig + 4 * m))  # at least one whole run of m positions
    if kv == KV_F16 and rng.integers(0, 4) == 0:  # record rebuilt at compression time
        record = B.SC_RECORD_RECOMPUTE
        w = int(rng.integers(1, 300))
        prompt = int(rng.integers(2 * m, n_trig))   # (the prompt itself then holds no compression)
    decode = int(rng.integers(m + 2, 2 * m + 30))
    wl = Workload("dense-%d" % seed, 700 + seed, int(rng.integers(1, 3)), int(rng.integers(1, 4)), d, kv,
                  prompt, decode, budget, r, w, m, float(rng.choice([0.0, 0.05])))
    return wl, trigger, thresh, record


@pytest.mark.parametrize("seed", range(30))
def test_random_dense_prefill_matches_oracle(seed):
    wl, trigger, thresh, record = _draw_dense(seed)
    print("\n", wl, "trigger", trigger, "thresh", thresh, "record", record, flush=True)
    run = ParityRun(wl, trigger=trigger, thresh=thresh, record_mode=record)
    plan = B.sc_prefill_plan(run.cfg, wl.prompt)
    assert any(dense for _, dense, _ in plan)
    run.prefill(wl.prompt)
    st = run.run()
    assert st["steps"] == wl.total


def _draw_i4_variants(seed):
    """4-bit rows (128 channels, every third seed 64) with the records that are not bucket counters: the exact ring
    (dense prompt runs write bits) or the record rebuilt at compression time."""
    rng = np.random.default_rng(9000 + seed)
    m = int(rng.integers(16, 160))
    budget = int(rng.integers(2 * m, 2 * m + 300))
    trigger = int(rng.choice([B.SC_TRIGGER_HARD_CAP, B.SC_TRIGGER_HIGH_WATER]))
    n_trig = budget + 1 if trigger == B.SC_TRIGGER_HARD_CAP else budget + m
    r = int(rng.integers(1, n_trig - m))
    w = int(rng.integers(1, 300))
    thresh = int(rng.choice([B.SC_THRESH_INV_POS, B.SC_THRESH_INV_LEN]))
    if rng.integers(0, 2) == 0:
        record, window = B.SC_RECORD_ONLINE, B.SC_WINDOW_RING
        prompt = int(rng.integers(2 * m, n_trig + 4 * m))
    else:
        record, window = B.SC_RECORD_RECOMPUTE, B.SC_WINDOW_AUTO
        prompt = int(rng.integers(2 * m, n_trig))
    decode = int(rng.integers(m + 2, 2 * m + 30))
    wl = Workload("i4var-%d" % seed, 900 + seed, int(rng.integers(1, 3)), int(rng.integers(1, 4)),
                  128 if seed % 3 else 64, KV_I4G64, prompt, decode, budget, r, w, m,
                  float(rng.choice([0.0, 0.05])))
    return wl, trigger, thresh, window, record


@pytest.mark.parametrize("seed", range(20))
def test_random_4bit_ring_and_recompute_match_oracle(seed):
    wl, trigger, thresh, window, record = _draw_i4_variants(seed)
    print("\n", wl, "trigger", trigger, "thresh", thresh, "window", window, "record", record, flush=True)
    run = ParityRun(wl, trigger=trigger, thresh=thresh, window_mode=window, record_mode=record)
    assert any(dense for _, dense, _ in B.sc_prefill_plan(run.cfg, wl.prompt))
    run.prefill(wl.prompt)
    st = run.run()
    assert st["steps"] == wl.total
