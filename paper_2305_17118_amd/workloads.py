"""Seeded synthetic inputs for the budgeted-KV-cache decode path.

This module is the only code shared by the GPU tests/benchmark and the CPU oracle.  It
holds no arithmetic of the method itself: it only draws the query/key/value streams.

The paper evaluates on trained OPT models over public text corpora; neither is available
offline, so the streams below stand in for them: OPT head shapes, N(0,1) entries, and,
for the larger configurations, a seeded set of "heavy hitter" positions whose keys carry
a fixed bias along a direction the queries share, so that a few rows keep receiving high
attention at every step (the repetitive pattern of Sec. 3.1 and the power-law scores
assumed in Sec. 4.2).

Recipe, per unit ``u`` (one sequence-head pair), all draws from
``numpy.random.Generator(Philox(key=[seed, u]))`` in this order:
  1. ``dir``  : d normals, normalised to unit length            (always drawn)
  2. ``q``    : [T, d] normals (float32 draws)
  3. ``k``    : [T, d] normals
  4. ``v``    : [T, d] normals
  5. ``perm`` : permutation of T; the first round(heavy_frac*T) entries are heavy rows
then, when heavy_frac > 0:  q += sqrt(d)*dir ;  k[heavy] += heavy_bias*dir.
With scale 1/sqrt(d) a heavy row's logit is shifted by +heavy_bias at every step.
Values are finally cast to the storage input type (float32, or float16).
Units are independent, so any subset can be generated without the rest.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np

KV_F32, KV_F16, KV_I4G64 = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    batch: int
    heads: int
    head_dim: int
    kv_dtype: int
    prompt: int
    decode: int
    budget: int
    recent: int
    history: int
    drop: int
    heavy_frac: float = 0.0
    heavy_bias: float = 4.0

    @property
    def units(self) -> int:
        return self.batch * self.heads

    @property
    def total(self) -> int:
        return self.prompt + self.decode

    @property
    def seed(self) -> int:
        return 20230517 + self.config_id

    @property
    def in_dtype(self):
        return np.float32 if self.kv_dtype == KV_F32 else np.float16

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five configurations the throughput metric is defined on (index 0 is the small case
# the oracle finishes in seconds; index 1 is the one the headline number is quoted on).
CONFIGS = (
    Workload("cfg1-small-fp32", 1, 1, 12, 64, KV_F32, 512, 128, 256, 32, 64, 64),
    Workload("cfg2-opt6.7b-fp16", 2, 16, 32, 128, KV_F16, 1024, 1024, 1024, 64, 256, 128),
    Workload("cfg3-opt13b-fp16", 3, 64, 40, 128, KV_F16, 2048, 256, 410, 64, 256, 128, 0.05),
    Workload("cfg4-opt66b-fp16", 4, 128, 72, 128, KV_F16, 2048, 128, 683, 128, 512, 256, 0.03),
    Workload("cfg5-opt175b-int4", 5, 32, 96, 128, KV_I4G64, 2048, 256, 683, 128, 512, 256, 0.05),
)


def unit_streams(wl: Workload, unit: int, steps: int | None = None):
    """q, k, v of one unit, each [T, d] in the workload's input dtype.

    ``steps`` truncates the returned stream (the draws themselves always cover the full
    length, so a prefix equals the prefix of the full stream)."""
    T, d = wl.total, wl.head_dim
    if steps is not None and steps > T:
        raise ValueError("workload %s has %d positions, %d asked for" % (wl.name, T, steps))
    rng = np.random.Generator(np.random.Philox(key=[wl.seed, unit]))
    direction = rng.standard_normal(d)
    direction /= np.linalg.norm(direction)
    q = rng.standard_normal((T, d), dtype=np.float32)
    k = rng.standard_normal((T, d), dtype=np.float32)
    v = rng.standard_normal((T, d), dtype=np.float32)
    perm = rng.permutation(T)
    if wl.heavy_frac > 0.0:
        heavy = perm[: int(round(wl.heavy_frac * T))]
        dvec = direction.astype(np.float32)
        q += np.float32(np.sqrt(d)) * dvec
        k[heavy] += np.float32(wl.heavy_bias) * dvec
    if steps is not None:
        q, k, v = q[:steps], k[:steps], v[:steps]
    dt = wl.in_dtype
    return q.astype(dt), k.astype(dt), v.astype(dt)


def streams(wl: Workload, units=None, steps: int | None = None, threads: int = 8):
    """q, k, v for the listed units (default: all), each [len(units), T, d]."""
    units = list(range(wl.units)) if units is None else [int(u) for u in units]
    T = wl.total if steps is None else steps
    shape = (len(units), T, wl.head_dim)
    q = np.empty(shape, dtype=wl.in_dtype)
    k = np.empty(shape, dtype=wl.in_dtype)
    v = np.empty(shape, dtype=wl.in_dtype)

    def fill(i):
        q[i], k[i], v[i] = unit_streams(wl, units[i], steps)

    if len(units) <= 2 or threads <= 1:
        for i in range(len(units)):
            fill(i)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(len(units))))
    return q, k, v


def sample_units(wl: Workload, count: int) -> list[int]:
    """A seeded, sorted sample of unit indices (always contains unit 0 and the last)."""
    U = wl.units
    if count >= U:
        return list(range(U))
    count = max(count, 2)
    rng = np.random.Generator(np.random.Philox(key=[wl.seed, 0xFFFF_FFFF]))
    inner = rng.choice(np.arange(1, U - 1), size=count - 2, replace=False).tolist()
    return sorted([0, U - 1] + inner)
