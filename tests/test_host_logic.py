"""Host-side logic of the C-ABI library (no GPU needed): exported symbols, configuration
checks, derived sizes, and the counter-bucket schedule that must reproduce the history window
of Alg. 2 at every compression step."""
import ctypes
import os
import re

import pytest

from paper_2305_17118_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(**kw):
    base = dict(batch=2, heads=4, head_dim=128, kv_dtype=B.SC_KV_F16, budget=64, recent=8,
                history=32, drop=16)
    base.update(kw)
    return B.make_config(**base)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "sc.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(sc_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS), (declared ^ set(B.EXPORTS))
    raw = ctypes.CDLL(B.LIB_PATH)
    for name in sorted(declared):
        assert getattr(raw, name) is not None


def test_status_strings():
    seen = {B.sc_status_str(s) for s in range(9)}
    assert len(seen) == 9 and "ok" in seen
    assert B.sc_status_str(99) == "unknown status"


@pytest.mark.parametrize("trigger,expect", [(B.SC_TRIGGER_HARD_CAP, 65), (B.SC_TRIGGER_HIGH_WATER, 80)])
def test_sizes(trigger, expect):
    n_trig, cap, E, W32 = B.sc_config_sizes(_cfg(trigger=trigger))
    assert n_trig == expect and cap == 128 and E == 2 and W32 == 0
    assert cap % 64 == 0 and cap >= n_trig


def test_workspace_accounts_for_every_array():
    for kv, row in ((B.SC_KV_F32, 512), (B.SC_KV_F16, 256), (B.SC_KV_I4G64, 64 + 8)):
        cfg = _cfg(kv_dtype=kv)
        _, cap, E, _ = B.sc_config_sizes(cfg)
        U = 8
        need = U * cap * (2 * row + 4 + 2 * E + 4) + U * 4
        got = B.sc_workspace_bytes(cfg)
        assert need <= got <= need + 10 * 256


@pytest.mark.parametrize("kw,status", [
    (dict(head_dim=96), B.SC_ERR_UNSUPPORTED),
    (dict(kv_dtype=7), B.SC_ERR_UNSUPPORTED),
    (dict(history=9000), B.SC_ERR_UNSUPPORTED),    # window longer than the build covers
    (dict(window_mode=5), B.SC_ERR_INVALID_ARG),
    (dict(budget=16, recent=16, drop=16, history=16), B.SC_ERR_INVALID_ARG),  # m > n_trig - r
    (dict(batch=0), B.SC_ERR_INVALID_ARG),
    (dict(recent=0), B.SC_ERR_INVALID_ARG),
    (dict(drop=0), B.SC_ERR_INVALID_ARG),
    (dict(trigger=3), B.SC_ERR_INVALID_ARG),
    (dict(thresh_mode=-1), B.SC_ERR_INVALID_ARG),
    (dict(scale=-1.0), B.SC_ERR_INVALID_ARG),
])
def test_bad_configs(kw, status):
    cfg = _cfg(**kw)
    with pytest.raises(B.ScError) as e:
        B.sc_config_sizes(cfg)
    assert e.value.status == status
    assert B.sc_workspace_bytes(cfg) == 0


def test_create_rejects_bad_workspace_without_touching_the_gpu():
    cfg = _cfg()
    need = B.sc_workspace_bytes(cfg)
    with pytest.raises(B.ScError) as e:
        B.sc_cache_create(cfg, 0, need)
    assert e.value.status == B.SC_ERR_INVALID_ARG
    with pytest.raises(B.ScError) as e:
        B.sc_cache_create(cfg, 4096, need - 1)
    assert e.value.status == B.SC_ERR_WORKSPACE
    with pytest.raises(B.ScError) as e:
        B.sc_cache_create(cfg, 4096 + 16, need)
    assert e.value.status == B.SC_ERR_WORKSPACE


@pytest.mark.parametrize("B_,r,w,m,trigger", [
    (256, 32, 64, 64, 0), (1024, 64, 256, 128, 0), (410, 64, 256, 128, 0), (683, 128, 512, 256, 1),
    (20, 2, 12, 3, 0), (20, 2, 12, 3, 1), (9, 1, 5, 1, 0), (30, 4, 40, 8, 0),
])
def test_bucket_schedule_reproduces_the_history_window(B_, r, w, m, trigger):
    """Simulate which steps each bucket holds.  At every compression step T_k the union of the
    buckets must be exactly the last w steps (T_k - w, T_k] (those that exist), and the bucket
    cleared after the compression must be the one holding the oldest epoch."""
    cfg = _cfg(budget=B_, recent=r, history=w, drop=m, trigger=trigger)
    n_trig, _, E, _ = B.sc_config_sizes(cfg)
    assert E == w // m
    buckets = [set() for _ in range(E)]
    n = 0
    compressions = 0
    for t in range(1, n_trig + 6 * m + 3):
        epoch, b, counted = B.sc_schedule(cfg, t)
        if counted:
            buckets[b].add(t)
        n += 1
        if n == n_trig:
            assert t == n_trig + compressions * m and epoch == compressions
            held = set().union(*buckets)
            assert held == set(range(max(1, t - w + 1), t + 1))
            nxt_epoch, nxt_bucket, _ = B.sc_schedule(cfg, t + 1)
            assert nxt_epoch == epoch + 1
            # everything in the bucket that will be reused has left the next window
            assert all(s <= t + m - w for s in buckets[nxt_bucket])
            buckets[nxt_bucket].clear()
            n -= m
            compressions += 1
    assert compressions >= 6


@pytest.mark.parametrize("w,m,mode", [(40, 16, 0), (400, 512, 0), (33, 8, 0), (32, 16, 1), (7, 5, 0)])
def test_ring_mode_sizes_and_schedule(w, m, mode):
    """A window that is not a multiple of the drop amount (the paper's own w = 400 with
    m = 0.5 B is one) selects the exact ring: ceil(w/32) words per row, every step counted,
    step t owns bit t mod w."""
    cfg = _cfg(budget=1024, recent=10, history=w, drop=m, window_mode=mode)
    _, cap, E, W32 = B.sc_config_sizes(cfg)
    assert E == 0 and W32 == (w + 31) // 32
    bucket_cfg = _cfg(budget=1024, recent=10, history=m * 2, drop=m)
    assert B.sc_workspace_bytes(cfg) - B.sc_workspace_bytes(bucket_cfg) == 8 * cap * (4 * W32 - 4)
    for t in (1, 2, w - 1, w, w + 1, 5 * w + 3):
        _, word, counted = B.sc_schedule(cfg, t)
        assert counted and word == (t % w) // 32


def test_kv_cache_accounting_matches_the_papers_table():
    rows = []
    for line in open(os.path.join(ROOT, "tests", "golden", "kv_cache_table1.txt")):
        if line.strip() and not line.startswith("#"):
            name, layers, d_model, gb = line.split()
            rows.append((name, int(layers), int(d_model), int(gb)))
    got = {name: B.kv_cache_bytes(L, d, batch=128, seq=2048) / 2 ** 30 for name, L, d, _ in rows}
    printed = {name: gb for name, _, _, gb in rows}
    assert got["OPT-175B"] == printed["OPT-175B"] == 1152
    assert got["LLaMA-65B"] == printed["LLaMA-65B"] == 640
    assert got["BLOOM"] == 980  # the paper prints 950 for this row


def test_compression_ratio_of_the_workloads():
    """Budget / full length gives the compression labels of the five workloads."""
    from paper_2305_17118_amd.workloads import CONFIGS
    ratios = [round(2048 / c.budget) for c in CONFIGS]
    assert ratios[1:] == [2, 5, 3, 3]


@pytest.mark.parametrize("kw,prompt", [
    (dict(), 500),
    (dict(budget=410, recent=64, history=256, drop=128), 2048),
    (dict(budget=1024, recent=64, history=256, drop=128), 1024),          # never reaches the trigger
    (dict(trigger=B.SC_TRIGGER_HIGH_WATER), 333),
    (dict(budget=60, recent=4, history=16, drop=4), 150),                 # runs too short for a dense block
    (dict(kv_dtype=B.SC_KV_I4G64), 200),
    (dict(kv_dtype=B.SC_KV_F32, head_dim=64), 200),                       # no dense kernel for fp32 rows
    (dict(history=40), 200),                                              # ring record, fp16: dense too
    (dict(history=40, kv_dtype=B.SC_KV_I4G64), 200),                      # ring record, 4-bit: dense too
    (dict(history=40, kv_dtype=B.SC_KV_I4G64, head_dim=64), 200),         # 4-bit rows of 64 channels too
    (dict(kv_dtype=B.SC_KV_F32, head_dim=64), 200),                       # fp32 rows (fp32 matrix instruction)
])
def test_prefill_plan_follows_the_schedule(kw, prompt):
    """The runs sc_prefill cuts a prompt into, against a position-by-position simulation of
    Alg. 1: runs tile the prompt, every position of a run falls into the same counter epoch, a
    compression can only follow the last position of a run, and it follows exactly when the
    cache has reached its trigger size."""
    cfg = _cfg(**kw)
    n_trig, cap, E, W32 = B.sc_config_sizes(cfg)
    plan = B.sc_prefill_plan(cfg, prompt)
    assert sum(r[0] for r in plan) == prompt and all(r[0] >= 1 for r in plan)
    dense_capable = E > 0 or W32 > 0
    t = n = 0
    for length, dense, compress in plan:
        epochs = {B.sc_schedule(cfg, t + 1 + i)[0] for i in range(length)}
        assert len(epochs) == 1
        for i in range(length):
            t += 1
            n += 1
            assert n <= n_trig
            if i < length - 1:
                assert n < n_trig  # no compression inside a run
        assert compress == (n == n_trig)
        if compress:
            n -= cfg.drop
        assert dense == (dense_capable and length >= 16)
    streamed = B.sc_prefill_plan(cfg, prompt, B.SC_PREFILL_STREAMED)
    assert [r[0] for r in streamed] == [r[0] for r in plan] and not any(r[1] for r in streamed)


def test_prefill_plan_rejects_bad_arguments():
    cfg = _cfg()
    with pytest.raises(B.ScError) as e:
        B.sc_prefill_plan(cfg, 0)
    assert e.value.status == B.SC_ERR_INVALID_ARG
    with pytest.raises(B.ScError) as e:
        B.sc_prefill_plan(cfg, 10, 7)
    assert e.value.status == B.SC_ERR_INVALID_ARG


def test_recomputed_record_configuration():
    """Record rebuilt at compression time: one 16-bit count per slot, a ring of w queries in the
    workspace, any w (no bucket constraint), every storage type."""
    cfg = _cfg(record_mode=B.SC_RECORD_RECOMPUTE, history=37)
    n_trig, cap, E, W32 = B.sc_config_sizes(cfg)
    assert (E, W32) == (1, 0)
    online = _cfg(history=32)  # E = 2
    extra = B.sc_workspace_bytes(cfg) - B.sc_workspace_bytes(online)
    U = 8
    assert abs(extra - (U * 37 * 128 * 2 - U * cap * 2)) <= 4 * 256
    for kv in (B.SC_KV_F32, B.SC_KV_I4G64):
        for d in (64, 128):
            assert B.sc_config_sizes(_cfg(record_mode=B.SC_RECORD_RECOMPUTE, kv_dtype=kv, head_dim=d))[2:] == (1, 0)
    f32 = _cfg(record_mode=B.SC_RECORD_RECOMPUTE, history=37, kv_dtype=B.SC_KV_F32)  # fp32 queries: 4 bytes
    extra32 = B.sc_workspace_bytes(f32) - B.sc_workspace_bytes(_cfg(history=32, kv_dtype=B.SC_KV_F32))
    assert abs(extra32 - (U * 37 * 128 * 4 - U * cap * 2)) <= 4 * 256
    with pytest.raises(B.ScError) as e:
        B.sc_config_sizes(_cfg(record_mode=3))
    assert e.value.status == B.SC_ERR_INVALID_ARG


@pytest.mark.parametrize("kw", [
    dict(), dict(trigger=B.SC_TRIGGER_HIGH_WATER), dict(budget=20, recent=3, history=8, drop=1),
    dict(budget=50, recent=5, history=51, drop=23), dict(budget=9, recent=1, history=6, drop=9,
                                                         trigger=B.SC_TRIGGER_HIGH_WATER),
])
def test_rows_and_due_steps_follow_from_the_token_count(kw):
    """Ragged batches evaluate n_b and "compression due" on the device from t_b alone; that closed
    form must equal the state machine of Alg. 1 (append one row per step, drop m whenever the
    trigger size is reached) at every step, and agree with sc_schedule about the buckets."""
    cfg = _cfg(**kw)
    n_trig = B.sc_config_sizes(cfg)[0]
    n = 0
    for t in range(1, 6 * n_trig):
        n += 1
        rows, due = B.sc_schedule_rows(cfg, t)
        assert rows == n and due == (n == n_trig), (t, rows, n, due)
        if due:
            n -= cfg.drop
    with pytest.raises(B.ScError):
        B.sc_schedule_rows(cfg, 0)


def test_layer_set_workspace_is_the_sum_of_its_layers():
    """Per-layer budgets (Sec. 4.1, budgets across layers): the set's workspace is the layers'
    workspaces back to back; an invalid layer makes the whole set invalid."""
    cfg = _cfg()
    budgets, drops = [32, 64, 96, 200], [16, 32, 48, 100]
    lib = B.lib()
    arr = lambda xs: (ctypes.c_int32 * len(xs))(*xs)
    total = lib.sc_layers_workspace_bytes(ctypes.byref(cfg), 4, arr(budgets), arr(drops))
    assert total == sum(B.sc_workspace_bytes(_cfg(budget=b, drop=m)) for b, m in zip(budgets, drops))
    same_drop = lib.sc_layers_workspace_bytes(ctypes.byref(cfg), 2, arr([64, 128]), None)
    assert same_drop == B.sc_workspace_bytes(_cfg(budget=64)) + B.sc_workspace_bytes(_cfg(budget=128))
    assert lib.sc_layers_workspace_bytes(ctypes.byref(cfg), 2, arr([64, 0]), None) == 0
    assert lib.sc_layers_workspace_bytes(ctypes.byref(cfg), 0, arr([64]), None) == 0
    assert lib.sc_layers_count(None) == 0 and not lib.sc_layers_get(None, 0)


def test_header_is_plain_c(tmp_path):
    """include/sc.h is the boundary: it must compile as C99 on its own (no C++, no HIP or torch
    types), and every declared function must be callable with the documented argument types."""
    import shutil
    import subprocess

    if shutil.which("gcc") is None:
        pytest.skip("needs gcc")
    src = tmp_path / "use_sc.c"
    src.write_text(
        '#include "sc.h"\n'
        "int use(void) {\n"
        "    sc_config cfg = {1, 1, 64, SC_KV_F16, 8, 1, 4, 2, SC_TRIGGER_HARD_CAP, SC_THRESH_INV_POS,\n"
        "                     SC_WINDOW_AUTO, SC_RECORD_ONLINE, 0.0f};\n"
        "    int32_t a, b, c, d;\n"
        "    sc_cache *h = 0;\n"
        "    sc_layers *ls = 0;\n"
        "    int32_t lens[1] = {3};\n"
        "    uint8_t act[1] = {1};\n"
        "    if (sc_config_sizes(&cfg, &a, &b, &c, &d) != SC_OK) return 1;\n"
        "    if (sc_cache_create(&cfg, 0, sc_workspace_bytes(&cfg), 0, &h) == SC_OK) return 2;\n"
        "    (void)sc_prefill_ragged(h, 0, 0, 0, lens, 0, 0, 0, SC_PREFILL_AUTO, 0);\n"
        "    (void)sc_decode_step_ragged(h, 0, 0, 0, 0, 0, 0, act, &a, 0);\n"
        "    (void)sc_compress_ragged(h, 0, 0, 0);\n"
        "    (void)sc_layers_create(&cfg, 1, lens, 0, 0, 0, 0, &ls);\n"
        "    return sc_status_str(SC_ERR_FULL) != 0;\n"
        "}\n")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
