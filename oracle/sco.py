"""ctypes front end of the CPU oracle (``sco.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module and this
module never imports the product package.

``Oracle`` mirrors the steps of Alg. 1 / Alg. 2 of the paper (append, budgeted attention
of Sec. 4.1, online importance record, compression); see the header of ``sco.c`` for the
readings taken.  Inputs are numpy arrays: fp32 for fp32 storage, float16 otherwise.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sco.c")
_LIB = os.path.join(_HERE, "libsco.so")

F32, F16, I4G64 = 0, 1, 2
HARD_CAP, HIGH_WATER = 0, 1
INV_POS, INV_LEN = 0, 1
RECORD_ONLINE, RECORD_RECOMPUTE = 0, 1


def build(force: bool = False) -> str:
    """Compile ``sco.c`` with gcc into ``libsco.so`` beside it (plain -O2, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-pthread",
               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


class _Cfg(C.Structure):
    _fields_ = [(k, C.c_int32) for k in (
        "batch", "heads", "head_dim", "kv_dtype", "budget", "recent", "history", "drop",
        "trigger", "thresh_mode")] + [("scale", C.c_double), ("record_mode", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        l = C.CDLL(build())
        l.sco_create.restype = C.c_void_p
        l.sco_create.argtypes = [C.POINTER(_Cfg), C.c_int]
        l.sco_destroy.argtypes = [C.c_void_p]
        l.sco_len.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int64),
                              C.POINTER(C.c_int32)]
        l.sco_step.argtypes = [C.c_void_p] + [C.c_void_p] * 6 + [C.c_int, C.POINTER(C.c_int32)]
        l.sco_compress.argtypes = [C.c_void_p, C.c_void_p]
        l.sco_compress_recompute.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                             C.c_void_p]
        l.sco_importance.argtypes = [C.c_void_p, C.c_void_p]
        l.sco_importance_online.argtypes = [C.c_void_p, C.c_void_p]
        l.sco_positions.argtypes = [C.c_void_p, C.c_void_p]
        l.sco_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        l.sco_i4_roundtrip.argtypes = [C.c_void_p, C.c_int] + [C.c_void_p] * 4
        l.sco_half_to_float.restype = C.c_float
        l.sco_half_to_float.argtypes = [C.c_uint16]
        l.sco_float_to_half.restype = C.c_uint16
        l.sco_float_to_half.argtypes = [C.c_float]
        _lib = l
    return _lib


@dataclass
class OracleConfig:
    batch: int
    heads: int
    head_dim: int
    kv_dtype: int
    budget: int
    recent: int
    history: int
    drop: int
    trigger: int = HARD_CAP
    thresh_mode: int = INV_POS
    scale: float = 0.0
    record_mode: int = RECORD_ONLINE


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Oracle:
    """One budgeted KV cache over ``batch*heads`` independent units, on the CPU."""

    def __init__(self, cfg: OracleConfig, nthreads: int | None = None):
        self.cfg = cfg
        self.nthreads = int(nthreads or os.cpu_count() or 1)
        c = _Cfg(cfg.batch, cfg.heads, cfg.head_dim, cfg.kv_dtype, cfg.budget, cfg.recent,
                 cfg.history, cfg.drop, cfg.trigger, cfg.thresh_mode, float(cfg.scale),
                 cfg.record_mode)
        self._h = lib().sco_create(C.byref(c), self.nthreads)
        if not self._h:
            raise ValueError("oracle rejected the configuration: %r" % (cfg,))
        self.U = cfg.batch * cfg.heads
        self.d = cfg.head_dim
        self.in_dtype = np.float32 if cfg.kv_dtype == F32 else np.float16
        _, _, self.cap = self.lengths()

    def __del__(self):
        h = getattr(self, "_h", None)
        if h:
            lib().sco_destroy(h)
            self._h = None

    def lengths(self):
        n, t, cap = C.c_int32(), C.c_int64(), C.c_int32()
        lib().sco_len(self._h, C.byref(n), C.byref(t), C.byref(cap))
        return n.value, t.value, cap.value

    @property
    def n(self):
        return self.lengths()[0]

    @property
    def t(self):
        return self.lengths()[1]

    def _inp(self, a):
        a = np.ascontiguousarray(a, dtype=self.in_dtype).reshape(self.U, self.d)
        return a

    def step(self, q, k_new, v_new, p_forced=None, want_probs=True):
        """Append (k_new, v_new), attend with q.  Returns (out [U,d] f64, probs [U,cap] f64
        or None, due).  ``p_forced`` [U, >=n] fp32 replaces the oracle's own probabilities
        in the low-score decision only."""
        q, k_new, v_new = self._inp(q), self._inp(k_new), self._inp(v_new)
        out = np.empty((self.U, self.d), dtype=np.float64)
        probs = np.empty((self.U, self.cap), dtype=np.float64) if want_probs else None
        ld = 0
        if p_forced is not None:
            p_forced = np.ascontiguousarray(p_forced, dtype=np.float32)
            assert p_forced.ndim == 2 and p_forced.shape[0] == self.U
            ld = p_forced.shape[1]
        due = C.c_int32(0)
        rc = lib().sco_step(self._h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), _ptr(probs),
                            _ptr(p_forced), ld, C.byref(due))
        if rc:
            raise RuntimeError("sco_step refused the call (step while a compression is due?)")
        return out, probs, bool(due.value)

    def compress(self):
        """Alg. 2.  Returns the evicted slots [U, m] (ascending, pre-compaction numbering)."""
        ev = np.empty((self.U, self.cfg.drop), dtype=np.int32)
        rc = lib().sco_compress(self._h, _ptr(ev))
        if rc:
            raise RuntimeError("sco_compress called while no compression is due")
        return ev

    def compress_recompute(self, p_forced=None, want_probs=True):
        """Alg. 2 in record mode "recompute".  Returns (evicted [U, m], probs [U, W, cap] f64 or
        None, record [U, n]) where W = min(w, t) replayed steps, oldest first.  ``p_forced``
        [U, W, >=n] fp32 replaces the oracle's probabilities in the low-score decision."""
        n, t, _ = self.lengths()
        W = min(self.cfg.history, t)
        ev = np.empty((self.U, self.cfg.drop), dtype=np.int32)
        probs = np.empty((self.U, W, self.cap), dtype=np.float64) if want_probs else None
        rec = np.empty((self.U, n), dtype=np.int32)
        ld = 0
        if p_forced is not None:
            p_forced = np.ascontiguousarray(p_forced, dtype=np.float32)
            assert p_forced.ndim == 3 and p_forced.shape[:2] == (self.U, W)
            ld = p_forced.shape[2]
        rc = lib().sco_compress_recompute(self._h, _ptr(ev), _ptr(probs), _ptr(p_forced), ld, _ptr(rec))
        if rc:
            raise RuntimeError("sco_compress_recompute refused the call (not due, or online mode)")
        return ev, probs, rec

    def importance(self):
        I = np.empty((self.U, self.n), dtype=np.int32)
        lib().sco_importance(self._h, _ptr(I))
        return I

    def importance_online(self):
        """The online record whatever the record mode."""
        I = np.empty((self.U, self.n), dtype=np.int32)
        lib().sco_importance_online(self._h, _ptr(I))
        return I

    def positions(self):
        p = np.empty((self.U, self.n), dtype=np.int64)
        lib().sco_positions(self._h, _ptr(p))
        return p

    def rows(self):
        n = self.n
        K = np.empty((self.U, n, self.d), dtype=np.float32)
        V = np.empty((self.U, n, self.d), dtype=np.float32)
        lib().sco_rows(self._h, _ptr(K), _ptr(V))
        return K, V


def i4_roundtrip(x_f16):
    """x_f16 [d] float16 -> (codes [d] u8, scale [d/64] f16, zero [d/64] f16, stored [d] f32)."""
    x = np.ascontiguousarray(x_f16, dtype=np.float16)
    d = x.shape[0]
    codes = np.empty(d, dtype=np.uint8)
    scale = np.empty(d // 64, dtype=np.float16)
    zero = np.empty(d // 64, dtype=np.float16)
    stored = np.empty(d, dtype=np.float32)
    rc = lib().sco_i4_roundtrip(_ptr(x), d, _ptr(codes), _ptr(scale), _ptr(zero), _ptr(stored))
    if rc:
        raise ValueError("head_dim must be a positive multiple of 64")
    return codes, scale, zero, stored
