"""Full-size parity: the five workloads of the throughput metric at their real shapes, in the
launch configuration the benchmark times, GPU (all units) against the oracle on a seeded
sample of units (all heads of the first sequence plus units scattered over the batch; units
are independent and identically distributed, so a sample checks every code path).  Every
step of prompt and decode is compared; records, evicted slots, positions and stored rows
must agree bit for bit at every compression.
"""
import pytest

from paper_2305_17118_amd import binding as B
from paper_2305_17118_amd.workloads import CONFIGS, KV_F16, KV_F32, KV_I4G64, Workload, sample_units

from .parity_util import ParityRun

pytestmark = pytest.mark.gpu


def _sample(wl, extra):
    if wl.units <= 64:
        return list(range(wl.units))
    first_seq = list(range(wl.heads))
    # the last units of a large batch are handed out by ticket rather than by workgroup index
    last = [wl.units - 1, wl.units - 2, wl.units - wl.units // 32]
    return sorted(set(first_seq) | set(sample_units(wl, extra)) | set(last))


@pytest.mark.parametrize("idx,extra", [(0, 0), (1, 16), (2, 24), (3, 24), (4, 24)],
                         ids=[c.name for c in CONFIGS])
def test_workload_matches_oracle(idx, extra):
    wl = CONFIGS[idx]
    sel = _sample(wl, extra)
    print("\n%s: %d units on the GPU, %d on the oracle" % (wl.name, wl.units, len(sel)), flush=True)
    run = ParityRun(wl, sel=sel)
    st = run.run(check_rows_every=3)
    print(st, flush=True)
    assert st["steps"] == wl.total
    expected = sum(1 for t in range(1, wl.total + 1)
                   if t >= wl.budget + 1 and (t - wl.budget - 1) % wl.drop == 0)
    assert st["compressions"] == expected
    assert run.cache.n <= wl.budget + 1


@pytest.mark.parametrize("kv,d,batch", [(KV_F32, 64, 96), (KV_F16, 128, 96), (KV_I4G64, 128, 96), (KV_I4G64, 64, 96),
                                       (KV_I4G64, 128, 24), (KV_I4G64, 64, 24)],
                         ids=["f32", "f16", "i4-d128", "i4-d64", "i4-d128-768-units", "i4-d64-768-units"])
def test_many_small_units_drawn_by_ticket(kv, d, batch):
    """2048 units and more.  fp32/fp16 rows: the last sixteenth of the units is not tied to a
    workgroup index (workgroups draw tickets for them, surplus workgroups return).  4-bit rows:
    one wave per unit, which writes its output without the merge through LDS (768 units: two
    waves per unit).  Small caches, every step compared on the first sequence, on scattered units
    and on units of the tail."""
    wl = Workload("tickets", 90, batch, 32, d, kv, 40, 50, 32, 4, 16, 8)
    assert wl.units >= 2048 or batch == 24
    tail = list(range(wl.units - wl.units // 16, wl.units, 37)) + [wl.units - 1]
    run = ParityRun(wl, sel=sorted(set(_sample(wl, 16)) | set(tail)))
    st = run.run(check_rows_every=1)
    assert st["steps"] == wl.total and st["compressions"] >= 6


def test_headline_workload_high_water_policy():
    """The trigger policy that leaves exactly B rows after each compression, on the headline
    shape (shortened stream: 1024 prompt + 320 decode, three compressions)."""
    wl = CONFIGS[1].scaled(decode=320)
    run = ParityRun(wl, sel=_sample(wl, 8), trigger=B.SC_TRIGGER_HIGH_WATER)
    st = run.run(check_rows_every=2)
    assert st["compressions"] == 2 and run.cache.n == wl.budget + (wl.total - wl.budget - wl.drop) % wl.drop


@pytest.mark.parametrize("idx,extra,decode", [(0, 0, 128), (1, 8, 160), (2, 8, 140), (3, 8, 128), (4, 8, 280)],
                         ids=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_dense_prefill_at_full_size(idx, extra, decode):
    """The prompt of a full-size workload (fp32, fp16, 4-bit) through one sc_prefill call (dense causal blocks
    on the matrix cores), every position compared on the sampled units; the decode steps that
    follow carry the records accumulated during the prompt into two compressions that must
    match bit for bit."""
    wl = CONFIGS[idx].scaled(decode=decode)
    sel = _sample(wl, extra)
    run = ParityRun(wl, sel=sel)
    run.prefill(wl.prompt)
    st = run.run(check_rows_every=2)
    print(st, flush=True)
    assert st["steps"] == wl.total


def test_recomputed_record_at_full_size():
    """Alg. 2 as printed on the headline shape: records rebuilt at compression time from the
    last 256 queries (dense prefill of the prompt, then 300 decode steps, three compressions)."""
    wl = CONFIGS[1].scaled(decode=300)
    run = ParityRun(wl, sel=_sample(wl, 8), record_mode=B.SC_RECORD_RECOMPUTE)
    run.prefill(wl.prompt)
    st = run.run(check_rows_every=2)
    print(st, flush=True)
    assert st["compressions"] == 3


def test_ragged_batch_at_full_size():
    """The headline shape with prompts of different lengths (the mix `bench.py --ragged` times:
    256 ... 1024 positions) through one sc_prefill_ragged call, then 400 decode steps with every
    sequence on its own clock; the shortest, a middle and the longest sequence (all their heads)
    are followed by their oracles at every position, step and compression."""
    from bench import ragged_prompt_lengths

    from .ragged_util import RaggedParityRun

    wl = CONFIGS[1]
    plens = ragged_prompt_lengths(wl)
    steps = 400
    run = RaggedParityRun(wl, plens, [0] * wl.batch, [steps] * wl.batch, check_seqs=[0, 7, wl.batch - 1])
    run.prefill()
    st = run.run()
    print(st, flush=True)
    assert st["seq_steps"] == steps * wl.batch and st["seq_compressions"] >= 12
