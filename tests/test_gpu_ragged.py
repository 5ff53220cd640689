"""Ragged batches through the C ABI (sc_prefill_ragged / sc_decode_step_ragged / sc_compress_ragged)
against one single-sequence oracle per batch entry."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2305_17118_amd import binding as B
from paper_2305_17118_amd.workloads import KV_F16, KV_F32, KV_I4G64, Workload, streams
from tests.ragged_util import RaggedParityRun

pytestmark = pytest.mark.gpu


def _wl(name, batch, heads, d, kv, budget, r, w, m, heavy=0.0, seed=1300):
    # the lengths are per sequence; the workload only has to offer enough stream positions
    return Workload(name, seed, batch, heads, d, kv, 0, 1024, budget, r, w, m, heavy)


CASES = [
    # workload, prompts, starts, decodes
    (_wl("rag-f16-d128", 4, 3, 128, KV_F16, 64, 8, 32, 16, 0.05), [40, 0, 97, 150], [0, 0, 0, 0], [90, 120, 60, 75]),
    (_wl("rag-f16-d64", 3, 2, 64, KV_F16, 50, 4, 20, 10), [5, 70, 33], [0, 10, 25], [80, 40, 60]),
    (_wl("rag-f32", 3, 2, 64, KV_F32, 40, 4, 16, 8), [0, 30, 61], [0, 0, 7], [70, 50, 40]),
    (_wl("rag-i4-d128", 4, 2, 128, KV_I4G64, 64, 8, 32, 16, 0.05), [200, 17, 0, 64], [0, 3, 0, 20], [50, 90, 100, 40]),
    (_wl("rag-i4-d64", 2, 3, 64, KV_I4G64, 40, 4, 16, 8), [10, 55], [0, 0], [60, 45]),
    (_wl("rag-drop-one", 3, 2, 128, KV_F16, 24, 2, 5, 1), [3, 30, 0], [0, 0, 12], [40, 30, 25]),
]


LONG_CASES = [
    # few units with long caches
    (_wl("rag-long-f16", 3, 4, 128, KV_F16, 330, 8, 64, 32, 0.05), [300, 40, 0], [0, 0, 10], [120, 150, 100]),
    (_wl("rag-long-f32", 2, 3, 64, KV_F32, 280, 6, 40, 20), [270, 5], [0, 0], [90, 110]),
    # capacity above 512 slots, one sequence nearly full and one nearly empty
    (_wl("rag-split-f16", 2, 3, 128, KV_F16, 520, 8, 64, 32, 0.05), [505, 60], [0, 0], [90, 120]),
]


@pytest.mark.parametrize("wl,prompts,starts,decodes", LONG_CASES, ids=[c[0].name for c in LONG_CASES])
@pytest.mark.parametrize("window", [B.SC_WINDOW_AUTO, B.SC_WINDOW_RING], ids=["buckets", "ring"])
def test_ragged_batch_of_few_units_with_long_caches(wl, prompts, starts, decodes, window):
    """Ragged batches of few units whose sequences hold hundreds of rows of very different counts."""
    run = RaggedParityRun(wl, prompts, starts, decodes, window_mode=window)
    run.prefill()
    st = run.run()
    assert st["seq_steps"] == sum(decodes) and st["seq_compressions"] >= 3


@pytest.mark.parametrize("wl,prompts,starts,decodes", CASES, ids=[c[0].name for c in CASES])
@pytest.mark.parametrize("trigger", [B.SC_TRIGGER_HARD_CAP, B.SC_TRIGGER_HIGH_WATER], ids=["cap", "hw"])
def test_ragged_batch_matches_per_sequence_oracles(wl, prompts, starts, decodes, trigger):
    """Prompts of different lengths through one sc_prefill_ragged call, then decode steps in which
    sequences join and leave at their own steps; every sequence is compared with its own oracle
    at every position and step, and each compression with that sequence's Alg. 2."""
    run = RaggedParityRun(wl, prompts, starts, decodes, trigger=trigger)
    run.prefill()
    st = run.run()
    assert st["seq_steps"] == sum(decodes) and st["seq_compressions"] >= 3


@pytest.mark.parametrize("kv,d", [(KV_F16, 128), (KV_I4G64, 128), (KV_F32, 64)], ids=["f16", "i4", "f32"])
def test_ragged_batch_with_ring_record_and_inverse_length_threshold(kv, d):
    wl = _wl("rag-ring", 3, 2, d, kv, 48, 6, 37, 12, 0.05)
    run = RaggedParityRun(wl, [20, 0, 75], [0, 5, 0], [70, 60, 50], thresh=B.SC_THRESH_INV_LEN,
                          window_mode=B.SC_WINDOW_RING)
    run.prefill()
    st = run.run()
    assert st["seq_compressions"] >= 3


@pytest.mark.parametrize("kv", [KV_F16, KV_I4G64], ids=["f16", "i4"])
def test_ragged_prompts_continue_sequences_that_are_not_empty(kv):
    """A second turn: after some decode steps a few sequences receive more prompt positions (of
    different lengths), the others none; then all decode again."""
    wl = _wl("rag-turns", 4, 2, 128, kv, 64, 8, 32, 16, 0.05)
    #                prompts            decode steps taken in two phases of 30 and 40
    run = RaggedParityRun(wl, [40, 0, 97, 20], [0, 0, 0, 0], [70 + 120, 70, 70 + 35, 70 + 120])
    run.prefill()
    for s in range(30):
        if run.step(s):
            run.compress()
    run.prefill(lengths=[120, 0, 35, 120])
    run.decodes = [70, 70, 70, 70]
    for s in range(30, 70):
        if run.step(s):
            run.compress()
    run.check_state()
    assert run.stats["seq_steps"] == 4 * 70 and run.stats["seq_compressions"] >= 8


@pytest.mark.parametrize("kv,d", [(KV_F16, 128), (KV_F16, 64), (KV_I4G64, 128)], ids=["f16", "f16-d64", "i4"])
@pytest.mark.parametrize("thresh", [B.SC_THRESH_INV_POS, B.SC_THRESH_INV_LEN], ids=["inv-t", "inv-n"])
def test_ragged_batch_with_recomputed_record(kv, d, thresh):
    """Alg. 2 as printed on a ragged batch: nothing is counted during the steps; each sequence
    keeps its own last w queries (prompt positions included) and replays them at its own
    compressions, over its own resident rows."""
    wl = _wl("rag-re", 4, 2, d, kv, 60, 6, 40, 20, 0.05)
    # prompts stay below the trigger size (61): compressions inside sc_prefill cannot be forced
    run = RaggedParityRun(wl, [30, 0, 55, 55], [0, 4, 0, 0], [110, 90, 70, 100], thresh=thresh,
                          record_mode=B.SC_RECORD_RECOMPUTE)
    run.prefill()
    st = run.run()
    assert st["seq_steps"] == 370 and st["seq_compressions"] >= 8


@pytest.mark.parametrize("kv,window", [(KV_F16, B.SC_WINDOW_AUTO), (KV_I4G64, B.SC_WINDOW_RING)],
                         ids=["f16", "i4-ring"])
def test_finished_sequence_is_replaced_by_a_new_request(kv, window):
    """Continuous batching: a sequence that has finished is emptied with sc_cache_reset_seq (while
    one of them even has a compression pending) and a new request is prefilled into its slot;
    the other sequences decode on undisturbed, before, between and after."""
    wl = _wl("rag-reuse", 3, 2, 128, kv, 40, 4, 24, 12, 0.05)
    # sequence 1 stops after 35 steps; a second request of 52 prompt positions then takes its slot
    run = RaggedParityRun(wl, [30, 20, 0], [0, 0, 0], [140, 35 + 52 + 60, 140], window_mode=window)
    run.prefill()
    run.decodes = [140, 35, 140]
    for s in range(45):          # sequence 1 is idle from step 35 on
        if run.step(s):
            run.compress()
    run.restart(1)
    run.prefill(lengths=[0, 52, 0])
    run.starts, run.decodes = [0, 45, 0], [140, 60, 140]
    for s in range(45, 140):
        if run.step(s):
            run.compress()
    run.check_state()
    assert run.stats["seq_compressions"] >= 15


def test_ragged_calls_with_equal_lengths_equal_the_lock_step_calls():
    """All sequences active with equal counters: the ragged calls must leave exactly the state and
    outputs of sc_decode_step / sc_compress (same kernels, per-sequence values derived on the device)."""
    wl = _wl("rag-eq", 3, 4, 128, KV_F16, 64, 8, 32, 16, 0.05)
    T = 150
    q, k, v = (torch.from_numpy(a).cuda() for a in streams(wl, steps=T))
    cfg = B.make_config(wl.batch, wl.heads, wl.head_dim, wl.kv_dtype, wl.budget, wl.recent, wl.history, wl.drop)
    a, b = B.BudgetCache(cfg), B.BudgetCache(cfg)
    U, d = wl.units, wl.head_dim
    oa = torch.empty(U, d, dtype=torch.float16, device="cuda")
    ob = torch.empty_like(oa)
    for s in range(T):
        due_a = a.decode_step(q[:, s], k[:, s], v[:, s], oa, in_stride=T * d)
        due_b = b.decode_step_ragged(q[:, s], k[:, s], v[:, s], ob, in_stride=T * d)
        assert torch.equal(oa, ob) and due_b == (wl.batch if due_a else 0)
        if due_a:
            a.compress()
            b.compress_ragged()
    n = a.n
    assert all(b.len_seq(i) == (a.n, a.t) for i in range(wl.batch))
    assert torch.equal(a.pos()[:, :n], b.pos()[:, :n]) and torch.equal(a.cnt(), b.cnt())
    Ka, Va = a.kv_rows()
    Kb, Vb = b.kv_rows()
    assert torch.equal(Ka[:, :n], Kb[:, :n]) and torch.equal(Va[:, :n], Vb[:, :n])


def test_ragged_state_machine_errors():
    wl = _wl("rag-err", 2, 2, 128, KV_F16, 16, 2, 8, 4)
    cfg = B.make_config(wl.batch, wl.heads, wl.head_dim, wl.kv_dtype, wl.budget, wl.recent, wl.history, wl.drop)
    c = B.BudgetCache(cfg)
    U, d = wl.units, wl.head_dim
    x = torch.randn(U, d, device="cuda").half()
    out = torch.empty_like(x)
    with pytest.raises(B.ScError) as e:  # nothing is due before the first ragged call
        c.compress_ragged()
    assert e.value.status == B.SC_ERR_STATE
    with pytest.raises(B.ScError) as e:
        c.decode_step_ragged(x, x, x, out, active=[0, 0])
    assert e.value.status == B.SC_ERR_INVALID_ARG
    for _ in range(17):  # sequence 0 alone reaches its trigger size (B + 1 = 17)
        due = c.decode_step_ragged(x, x, x, out, active=[1, 0])
    assert due == 1 and c.len_seq(0) == (17, 17) and c.len_seq(1) == (0, 0)
    with pytest.raises(B.ScError) as e:  # even a step of the other sequence has to wait
        c.decode_step_ragged(x, x, x, out, active=[0, 1])
    assert e.value.status == B.SC_ERR_FULL
    for call in (lambda: c.decode_step(x, x, x, out), lambda: c.compress(), lambda: c.n):
        with pytest.raises(B.ScError) as e:  # lock-step calls are closed once counters are per sequence
            call()
        assert e.value.status == B.SC_ERR_STATE
    c.compress_ragged()
    assert c.len_seq(0) == (13, 17)
    with pytest.raises(B.ScError) as e:
        c.compress_ragged()
    assert e.value.status == B.SC_ERR_STATE
    c.prefill_ragged(x, x, x, [1, 0])  # a prompt may continue a sequence that is not empty
    assert c.len_seq(0) == (14, 18)
    for _ in range(3):  # sequence 0 due again (14 + 3 = 17 rows) ...
        due = c.decode_step_ragged(x, x, x, out, active=[1, 0])
    assert due == 1
    c.reset_seq(0)      # ... and dropped with its compression pending: nothing is due any more
    assert c.len_seq(0) == (0, 0)
    with pytest.raises(B.ScError) as e:
        c.compress_ragged()
    assert e.value.status == B.SC_ERR_STATE
    assert c.decode_step_ragged(x, x, x, out, active=[1, 1]) == 0
    assert c.len_seq(0) == (1, 1) and c.len_seq(1) == (1, 1)
    with pytest.raises(B.ScError) as e:
        c.reset_seq(2)
    assert e.value.status == B.SC_ERR_INVALID_ARG
    c.reset()  # back to lock step, empty
    assert (c.n, c.t) == (0, 0)
    assert c.decode_step(x, x, x, out) is False
    torch.cuda.synchronize()


def _draw(seed):
    rng = np.random.default_rng(7000 + seed)
    kv = int(rng.choice([KV_F32, KV_F16, KV_F16, KV_I4G64, KV_I4G64]))
    d = 64 if kv == KV_F32 else int(rng.choice([64, 128]))
    m = int(rng.integers(1, 40))
    budget = int(rng.integers(2 * m + 2, 2 * m + 150))
    trigger = int(rng.choice([B.SC_TRIGGER_HARD_CAP, B.SC_TRIGGER_HIGH_WATER]))
    n_trig = budget + 1 if trigger == B.SC_TRIGGER_HARD_CAP else budget + m
    r = int(rng.integers(1, n_trig - m))
    ring = bool(rng.integers(0, 2))
    w = int(rng.integers(1, 200)) if ring else m * int(rng.integers(1, 4))
    batch = int(rng.integers(2, 6))
    heads = int(rng.integers(1, 4))
    prompts = [int(rng.integers(0, 2 * n_trig)) if rng.integers(0, 4) else 0 for _ in range(batch)]
    if max(prompts) == 0:
        prompts[0] = n_trig + 3
    starts = [int(rng.integers(0, 30)) if rng.integers(0, 2) else 0 for _ in range(batch)]
    decodes = [int(rng.integers(m + 2, 3 * m + 60)) for _ in range(batch)]
    thresh = int(rng.choice([B.SC_THRESH_INV_POS, B.SC_THRESH_INV_LEN]))
    wl = _wl("rag-rnd-%d" % seed, batch, heads, d, kv, budget, r, w, m, float(rng.choice([0.0, 0.05])), 1400 + seed)
    return wl, prompts, starts, decodes, trigger, thresh, (B.SC_WINDOW_RING if ring else B.SC_WINDOW_AUTO)


@pytest.mark.parametrize("seed", range(24))
def test_random_ragged_configuration_matches_oracle(seed):
    wl, prompts, starts, decodes, trigger, thresh, window = _draw(seed)
    print("\n", wl, "prompts", prompts, "starts", starts, "decodes", decodes, "trigger", trigger, "thresh",
          thresh, "window", window, flush=True)
    run = RaggedParityRun(wl, prompts, starts, decodes, trigger=trigger, thresh=thresh, window_mode=window)
    run.prefill()
    st = run.run()
    assert st["seq_steps"] == sum(decodes)


def test_layer_set_with_growing_budgets_matches_standalone_caches_and_oracle():
    """One cache per layer, later layers with larger budgets (Sec. 4.1, budgets across layers;
    m = B/2 per layer): every layer of the set behaves exactly like a standalone cache with that
    layer's configuration (bit for bit), and the last layer is checked against the oracle."""
    from tests.parity_util import ParityRun

    budgets, drops = [32, 64, 96], [16, 32, 48]
    base = _wl("layers", 2, 3, 128, KV_F16, 32, 8, 96, 16, 0.05)
    T = 260
    q, k, v = (torch.from_numpy(a).cuda() for a in streams(base, steps=T))
    cfg = B.make_config(base.batch, base.heads, base.head_dim, base.kv_dtype, 32, base.recent, base.history, 16)
    ls = B.LayerSet(cfg, budgets, drops)
    assert len(ls) == 3
    U, d = base.units, base.head_dim
    for l, (bud, m) in enumerate(zip(budgets, drops)):
        solo = B.BudgetCache(B.make_config(base.batch, base.heads, d, base.kv_dtype, bud, base.recent,
                                           base.history, m))
        layer = ls[l]
        assert (layer.n_trig, layer.capacity) == (solo.n_trig, solo.capacity)
        oa = torch.empty(U, d, dtype=torch.float16, device="cuda")
        ob = torch.empty_like(oa)
        comps = 0
        for s in range(T):
            due_a = layer.decode_step(q[:, s], k[:, s], v[:, s], oa, in_stride=T * d)
            due_b = solo.decode_step(q[:, s], k[:, s], v[:, s], ob, in_stride=T * d)
            assert due_a == due_b and torch.equal(oa, ob)
            if due_a:
                layer.compress()
                solo.compress()
                comps += 1
        assert comps >= 3 and (layer.n, layer.t) == (solo.n, solo.t)
        n = solo.n
        assert torch.equal(layer.pos()[:, :n], solo.pos()[:, :n]) and torch.equal(layer.cnt(), solo.cnt())
    # the layers did not disturb each other: layer 0 still holds what its own steps left
    first = B.BudgetCache(B.make_config(base.batch, base.heads, d, base.kv_dtype, 32, base.recent, base.history, 16))
    ob = torch.empty(U, d, dtype=torch.float16, device="cuda")
    for s in range(T):
        if first.decode_step(q[:, s], k[:, s], v[:, s], ob, in_stride=T * d):
            first.compress()
    n = first.n
    K0, V0 = ls[0].kv_rows()
    K1, V1 = first.kv_rows()
    assert torch.equal(K0[:, :n], K1[:, :n]) and torch.equal(V0[:, :n], V1[:, :n])
    ls.close()
    wl = Workload("layer-2", 1300, base.batch, base.heads, d, base.kv_dtype, 0, T, 96, base.recent, base.history, 48, 0.05)
    run = ParityRun(wl)
    run.run()


@pytest.mark.parametrize("seed", range(8))
def test_random_serving_trace_matches_oracle(seed):
    """A serving trace with continuous batching: requests with random prompt lengths arrive in free
    slots (their prompt sometimes handed over in two chunks), decode for a random number of
    steps, sit out steps at random, finish and are replaced; every sequence is followed by its
    own oracle through all of it."""
    rng = np.random.default_rng(8100 + seed)
    kv = int(rng.choice([KV_F16, KV_I4G64, KV_F32]))
    d = 64 if kv == KV_F32 else int(rng.choice([64, 128]))
    m = int(rng.integers(4, 24))
    budget = int(rng.integers(2 * m + 4, 2 * m + 60))
    ring = bool(rng.integers(0, 2))
    w = int(rng.integers(3, 90)) if ring else m * int(rng.integers(1, 4))
    r = int(rng.integers(1, budget - m))
    batch, heads = int(rng.integers(2, 5)), int(rng.integers(1, 4))
    wl = _wl("rag-serve-%d" % seed, batch, heads, d, kv, budget, r, w, m, 0.05, 1500 + seed)
    T = 900  # stream positions available per sequence slot
    run = RaggedParityRun(wl, [0] * batch, [0] * batch, [T] * batch,
                          trigger=int(rng.choice([B.SC_TRIGGER_HARD_CAP, B.SC_TRIGGER_HIGH_WATER])),
                          thresh=int(rng.choice([B.SC_THRESH_INV_POS, B.SC_THRESH_INV_LEN])),
                          window_mode=B.SC_WINDOW_RING if ring else B.SC_WINDOW_AUTO)
    print("\n", wl, "ring" if ring else "buckets", flush=True)
    remaining = [0] * batch   # decode steps the request in each slot still wants (0: slot free)
    requests = 0
    for step in range(160):
        for b in range(batch):
            if remaining[b] == 0 and rng.random() < 0.35 and run.consumed[b] < T - 330:
                if run.cache.len_seq(b) != (0, 0):
                    run.restart(b)
                plen = int(rng.integers(1, 2 * budget))
                lens = [0] * batch
                if plen > 3 and rng.random() < 0.5:   # the prompt arrives in two chunks
                    cut = int(rng.integers(1, plen))
                    lens[b] = cut
                    run.prefill(lengths=lens)
                    lens[b] = plen - cut
                else:
                    lens[b] = plen
                run.prefill(lengths=lens)
                remaining[b] = int(rng.integers(1, 70))
                requests += 1
        active = [remaining[b] > 0 and rng.random() < 0.9 for b in range(batch)]
        if run.step_active(active, step):
            run.compress()
        for b in range(batch):
            remaining[b] -= int(active[b])
    run.check_state()
    assert requests >= batch and run.stats["seq_steps"] > 100


@pytest.mark.parametrize("kv,budget,plens,start,T", [
    (KV_F16, 40, [30, 0, 17], 40, 260),
    (KV_I4G64, 40, [30, 0, 17], 40, 260),
    # capacity above 512 slots and six units: every unit's rows are shared by 8 workgroups whose
    # arrival counters must be back at zero for every replay
    (KV_F16, 520, [500, 470, 510], 512, 700),
], ids=["f16", "i4", "f16-long"])
def test_decode_step_replayed_from_a_graph_with_the_device_clock(kv, budget, plens, start, T):
    """With the step count kept on the device one captured sc_decode_step_ragged call is replayed
    for every step between compressions, and again after each (eager) compression, with the
    inputs rewritten in place; outputs and the final cache must equal, bit for bit, those of a
    twin cache stepped eagerly with the step count passed as an argument."""
    wl = _wl("rag-graph", 3, 2, 128, kv, budget, 4, 24, 12, 0.05)
    U, d = wl.units, wl.head_dim
    q, k, v = (torch.from_numpy(a).cuda() for a in streams(wl, steps=T))
    cfg = B.make_config(wl.batch, wl.heads, d, kv, wl.budget, wl.recent, wl.history, wl.drop)
    eager, graphed = B.BudgetCache(cfg), B.BudgetCache(cfg)
    for c in (eager, graphed):
        c.prefill_ragged(q, k, v, plens, T * d, None)
    graphed.device_clock(True)
    qs, ks, vs = (torch.empty(U, d, dtype=torch.float16, device="cuda") for _ in range(3))  # static inputs
    out_e = torch.empty(U, d, dtype=torch.float16, device="cuda")
    out_g = torch.empty_like(out_e)
    # `start`: stream position of the first decode step (past every prompt)

    def load(s):
        qs.copy_(q[:, s]); ks.copy_(k[:, s]); vs.copy_(v[:, s])

    # 1. an eager step brings the device table up to date
    load(start)
    assert eager.decode_step_ragged(qs, ks, vs, out_e) == graphed.decode_step_ragged(qs, ks, vs, out_g)
    assert torch.equal(out_e, out_g)
    # 2. capture one call (counted as a step; the first replay executes it)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        due_g = graphed.decode_step_ragged(qs, ks, vs, out_g)
    pending_first_replay = True
    comps = 0
    for s in range(start + 1, T):
        load(s)
        due_e = eager.decode_step_ragged(qs, ks, vs, out_e)
        if pending_first_replay:
            pending_first_replay = False
        else:
            assert graphed.steps_until_due() >= 1
            due_g = graphed.note_replays(1)
        g.replay()
        torch.cuda.synchronize()
        assert due_g == due_e and torch.equal(out_e, out_g), "step %d" % s
        if due_e:
            with pytest.raises(B.ScError) as e:
                graphed.note_replays(1)  # not past a due compression
            assert e.value.status == B.SC_ERR_FULL
            eager.compress_ragged()
            graphed.compress_ragged()   # eager; the same graph goes on afterwards
            comps += 1
    assert comps >= 10
    for b in range(wl.batch):
        assert eager.len_seq(b) == graphed.len_seq(b)
    assert torch.equal(eager.cnt(), graphed.cnt())
    Ka, Va = eager.kv_rows()
    Kb, Vb = graphed.kv_rows()
    for b in range(wl.batch):
        u, nb = slice(b * wl.heads, (b + 1) * wl.heads), eager.len_seq(b)[0]
        assert torch.equal(eager.pos()[u, :nb], graphed.pos()[u, :nb])
        assert torch.equal(Ka[u, :nb], Kb[u, :nb]) and torch.equal(Va[u, :nb], Vb[u, :nb])


def test_layer_set_step_in_one_call_and_replayed_from_one_graph():
    """sc_layers_decode_step = one sc_decode_step_ragged per layer: the layers of a set (own budgets
    and drop sizes, so compressions fall on different steps) are stepped (a) by one call per step
    and (b) by replaying ONE captured call, and must equal, bit for bit, standalone caches stepped
    layer by layer; compressions are eager in all three."""
    kv, L = KV_F16, 4
    wl = _wl("layers-graph", 2, 3, 128, kv, 40, 4, 24, 12, 0.05)
    T, U, d = 200, wl.units, wl.head_dim
    cfg = B.make_config(wl.batch, wl.heads, d, kv, wl.budget, wl.recent, wl.history, wl.drop)
    budgets, drops = [40, 46, 52, 64], [12, 12, 24, 8]
    q, k, v = (torch.from_numpy(a).cuda() for a in streams(wl.scaled(heads=wl.heads * L), steps=T))
    # [U*L, T, d] -> per layer [L, U, T, d]
    q, k, v = (x.view(wl.batch, L, wl.heads, T, d).permute(1, 0, 2, 3, 4).reshape(L, U, T, d).contiguous()
               for x in (q, k, v))
    import copy
    alone = []
    for l in range(L):
        c = copy.copy(cfg)
        c.budget, c.drop = budgets[l], drops[l]
        alone.append(B.BudgetCache(c))
    called, graphed = B.LayerSet(cfg, budgets, drops), B.LayerSet(cfg, budgets, drops)
    P = 20
    for l in range(L):
        for c in (alone[l], called[l], graphed[l]):
            c.prefill_ragged(q[l], k[l], v[l], [P] * wl.batch, T * d, None)
    graphed.device_clock(True)
    qs, ks, vs = (torch.empty(L, U, d, dtype=torch.float16, device="cuda") for _ in range(3))
    out_a, out_c, out_g = (torch.empty(L, U, d, dtype=torch.float16, device="cuda") for _ in range(3))

    def load(s):
        qs.copy_(q[:, :, s]); ks.copy_(k[:, :, s]); vs.copy_(v[:, :, s])

    def step_alone():
        return sum(alone[l].decode_step_ragged(qs[l], ks[l], vs[l], out_a[l]) for l in range(L))

    load(P)
    due = step_alone()
    assert called.decode_step(qs, ks, vs, out_c) == due == graphed.decode_step(qs, ks, vs, out_g)
    assert torch.equal(out_a, out_c) and torch.equal(out_a, out_g)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        due_g = graphed.decode_step(qs, ks, vs, out_g)
    first, comps = True, 0
    for s in range(P + 1, T):
        load(s)
        due = step_alone()
        assert called.decode_step(qs, ks, vs, out_c) == due
        if first:
            first = False
        else:
            assert graphed.steps_until_due() >= 1
            due_g = graphed.note_replays(1)
        g.replay()
        torch.cuda.synchronize()
        assert due_g == due, "step %d" % s
        assert torch.equal(out_a, out_c) and torch.equal(out_a, out_g), "step %d" % s
        if due:
            with pytest.raises(B.ScError) as e:
                graphed.note_replays(1)
            assert e.value.status == B.SC_ERR_FULL
            with pytest.raises(B.ScError) as e:
                called.decode_step(qs, ks, vs, out_c)
            assert e.value.status == B.SC_ERR_FULL
            n_alone = 0
            for c in alone:
                if any(c.len_seq(b)[0] == c.n_trig for b in range(wl.batch)):
                    c.compress_ragged()
                    n_alone += 1
            assert called.compress() == n_alone == graphed.compress()
            comps += n_alone
    assert comps >= 20
    with pytest.raises(B.ScError) as e:
        called.compress()
    assert e.value.status == B.SC_ERR_STATE
    for l in range(L):
        for other in (called[l], graphed[l]):
            assert torch.equal(alone[l].cnt(), other.cnt())
            Ka, Va = alone[l].kv_rows()
            Kb, Vb = other.kv_rows()
            for b in range(wl.batch):
                assert alone[l].len_seq(b) == other.len_seq(b)
                u, nb = slice(b * wl.heads, (b + 1) * wl.heads), alone[l].len_seq(b)[0]
                assert torch.equal(alone[l].pos()[u, :nb], other.pos()[u, :nb])
                assert torch.equal(Ka[u, :nb], Kb[u, :nb]) and torch.equal(Va[u, :nb], Vb[u, :nb])


def test_layer_set_calls_reject_bad_arguments_and_change_nothing():
    """Argument and state errors of the layer-set calls are found before anything is enqueued:
    strides that are too small or not 16-byte multiples, null pointers, a step or a replay
    without the device clock, a compression when none is due; the caches stay where they were."""
    kv, L = KV_F16, 3
    wl = _wl("layers-errors", 2, 2, 128, kv, 30, 4, 16, 8)
    U, d = wl.units, wl.head_dim
    cfg = B.make_config(wl.batch, wl.heads, d, kv, wl.budget, wl.recent, wl.history, wl.drop)
    ls = B.LayerSet(cfg, [30, 34, 38], [8, 8, 8])
    q, k, v = (torch.from_numpy(a).cuda() for a in streams(wl, steps=12))
    for l in range(L):
        ls[l].prefill_ragged(q, k, v, [10] * wl.batch, 12 * d, None)
    x = torch.zeros(L, U, d, dtype=torch.float16, device="cuda")
    out = torch.empty(L, U, d, dtype=torch.float16, device="cuda")
    lib, h, s = B.lib(), ls.handle, ls._stream()
    due = C.c_int32(-7)
    p, o = x.data_ptr(), out.data_ptr()
    before = [[ls[l].len_seq(b) for b in range(wl.batch)] for l in range(L)]

    def call(q_=p, k_=p, v_=p, ls_stride=U * d, in_stride=0, o_=o, out_stride=U * d):
        return lib.sc_layers_decode_step(h, q_, k_, v_, ls_stride, in_stride, o_, out_stride, None, C.byref(due), s)

    assert call(q_=None) == B.SC_ERR_INVALID_ARG and call(k_=None) == B.SC_ERR_INVALID_ARG
    assert call(v_=None) == B.SC_ERR_INVALID_ARG and call(o_=None) == B.SC_ERR_INVALID_ARG
    assert call(ls_stride=U * d - 8) == B.SC_ERR_INVALID_ARG       # layers would overlap
    assert call(ls_stride=U * d + 4) == B.SC_ERR_INVALID_ARG       # not a multiple of 16 bytes
    assert call(out_stride=U * d - 8) == B.SC_ERR_INVALID_ARG
    assert call(out_stride=U * d + 4) == B.SC_ERR_INVALID_ARG
    assert call(in_stride=2 * d) == B.SC_ERR_INVALID_ARG            # units 2d apart do not fit in U*d per layer
    assert lib.sc_layers_decode_step(None, p, p, p, U * d, 0, o, U * d, None, C.byref(due), s) == B.SC_ERR_INVALID_ARG
    assert due.value == -7
    with pytest.raises(B.ScError) as e:   # nothing captured to replay: the clock is off and no step was taken
        ls.note_replays(1)
    assert e.value.status == B.SC_ERR_STATE
    with pytest.raises(B.ScError) as e:
        ls.compress()
    assert e.value.status == B.SC_ERR_STATE
    torch.cuda.synchronize()
    assert before == [[ls[l].len_seq(b) for b in range(wl.batch)] for l in range(L)]
    assert call() == B.SC_OK and due.value == 0
    torch.cuda.synchronize()
    assert [[ls[l].len_seq(b) for b in range(wl.batch)] for l in range(L)] == \
        [[(n + 1, t + 1) for n, t in row] for row in before]
