"""sc_compress_static (the entry point that allocates nothing) against sc_compress.

Two caches of the same configuration receive the same seeded prompt and decode steps through
the C ABI; at every compression one calls sc_compress (scratch in the caller's workspace), the
other sc_compress_static (scratch in the library's own device array).  Evicted slots, positions,
records and stored rows must be identical bit for bit: it is integer and byte work.  Two runs
in a row share the library's array, the second with a smaller cache, so stale contents of the
first must not leak into the second.
"""
import numpy as np
import pytest
import torch

from paper_2305_17118_amd import binding as B
from paper_2305_17118_amd.workloads import KV_F16, KV_I4G64, Workload, streams

pytestmark = pytest.mark.gpu


def _pair_run(wl: Workload, record_mode=B.SC_RECORD_ONLINE):
    dev = torch.device("cuda:0")
    cfg = B.make_config(wl.batch, wl.heads, wl.head_dim, wl.kv_dtype, wl.budget, wl.recent, wl.history,
                        wl.drop, record_mode=record_mode)
    q, k, v = (torch.from_numpy(a).to(dev) for a in streams(wl, threads=8))
    ref, sta = B.BudgetCache(cfg, dev), B.BudgetCache(cfg, dev)
    U, d, T, m = wl.units, wl.head_dim, wl.total, wl.drop
    outs = [torch.empty(U, d, dtype=ref.io_dtype, device=dev) for _ in range(2)]
    evs = [torch.full((U, m), -1, dtype=torch.int32, device=dev) for _ in range(2)]
    compressions = 0
    for s in range(T):
        due = [c.decode_step(q[:, s], k[:, s], v[:, s], o, in_stride=T * d) for c, o in zip((ref, sta), outs)]
        assert due[0] == due[1]
        if due[0]:
            before = torch.cuda.memory_allocated(dev)
            ref.compress(evs[0])
            sta.compress_static(evs[1])
            assert torch.cuda.memory_allocated(dev) == before
            compressions += 1
            assert ref.n == sta.n == ref.n_trig - m
            n = ref.n
            assert torch.equal(evs[0], evs[1]), "evicted slots differ at step %d" % s
            assert torch.equal(ref.pos()[:, :n], sta.pos()[:, :n]), "positions differ at step %d" % s
            assert torch.equal(ref.cnt()[:, :, :ref.n_trig], sta.cnt()[:, :, :ref.n_trig]), "records differ"
            for a, b in zip(ref.kv_rows(), sta.kv_rows()):
                assert torch.equal(a[:, :n].view(torch.uint8), b[:, :n].view(torch.uint8)), "rows differ"
            if wl.kv_dtype == KV_I4G64:
                for a, b in zip(ref.kv_meta(), sta.kv_meta()):
                    assert torch.equal(a[:, :n].view(torch.int16), b[:, :n].view(torch.int16)), "meta differ"
        assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16)), "outputs differ at step %d" % s
    torch.cuda.synchronize()
    return compressions


def test_static_scratch_compress_matches_workspace_compress_twice_in_a_row():
    # several tiles of select/compact work per unit and a ragged tail; then a smaller cache
    big = Workload("noalloc-big", 71, 3, 5, 128, KV_F16, 0, 700, 300, 40, 128, 64, 0.05)
    small = Workload("noalloc-small", 72, 1, 3, 128, KV_I4G64, 0, 260, 70, 16, 48, 24, 0.05)
    assert _pair_run(big) >= 6
    assert _pair_run(small) >= 7


def test_static_scratch_compress_with_the_record_rebuilt_at_compression_time():
    wl = Workload("noalloc-replay", 73, 2, 2, 128, KV_F16, 0, 330, 120, 16, 100, 40, 0.05)
    assert _pair_run(wl, record_mode=B.SC_RECORD_RECOMPUTE) >= 5


def test_static_scratch_limit_and_state_errors():
    dev = torch.device("cuda:0")
    # 2048 units x 4160 slots x 4 bytes > 32 MiB
    cfg = B.make_config(16, 128, 64, KV_F16, 4100, 16, 64, 64)
    assert B.sc_config_sizes(cfg)[1] * 2048 * 4 > B.SC_STATIC_SCRATCH_BYTES
    c = B.BudgetCache(cfg, dev)
    with pytest.raises(B.ScError) as e:  # nothing is due on an empty cache: state comes first
        c.compress_static()
    assert e.value.status == B.SC_ERR_STATE
    U, d = 2048, 64
    x = torch.randn(U, 4101, d, device=dev).half()
    c.prefill(x, x, x, 4100, 4101 * d)
    out = torch.empty(U, d, dtype=torch.float16, device=dev)
    assert c.decode_step(x[:, 4100], x[:, 4100], x[:, 4100], out, in_stride=4101 * d)
    with pytest.raises(B.ScError) as e:
        c.compress_static()
    assert e.value.status == B.SC_ERR_SCRATCH
    assert c.n == c.n_trig  # unchanged; the workspace variant still serves
    c.compress()
    assert c.n == c.n_trig - 64
    torch.cuda.synchronize()
