"""ctypes binding of ``libsc.so`` (the C ABI of ``include/sc.h``), same names, marshalling only.

Device memory and streams come from PyTorch-ROCm: tensors are passed as ``data_ptr()`` and
the stream as ``torch.cuda.current_stream().cuda_stream``.  Nothing is computed here; if the
library is missing this module raises at first use, there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsc.so")

SC_OK, SC_ERR_INVALID_ARG, SC_ERR_WORKSPACE, SC_ERR_FULL, SC_ERR_STATE, SC_ERR_UNSUPPORTED, \
    SC_ERR_DEVICE, SC_ERR_SCRATCH, SC_ERR_HOST_MEMORY = range(9)
SC_STATIC_SCRATCH_BYTES = 32 << 20
SC_KV_F32, SC_KV_F16, SC_KV_I4G64 = 0, 1, 2
SC_TRIGGER_HARD_CAP, SC_TRIGGER_HIGH_WATER = 0, 1
SC_THRESH_INV_POS, SC_THRESH_INV_LEN = 0, 1
SC_WINDOW_AUTO, SC_WINDOW_RING = 0, 1
SC_PREFILL_AUTO, SC_PREFILL_STREAMED = 0, 1
SC_RECORD_ONLINE, SC_RECORD_RECOMPUTE = 0, 1

EXPORTS = (
    "sc_config_sizes", "sc_workspace_bytes", "sc_schedule", "sc_cache_create", "sc_cache_reset",
    "sc_cache_destroy",
    "sc_decode_step", "sc_compress", "sc_compress_static", "sc_prefill", "sc_prefill_plan", "sc_cache_len", "sc_cache_view", "sc_status_str",
    "sc_diag_persistence", "sc_diag_kept_mass", "sc_diag_trace", "sc_diag_read_bandwidth",
    "sc_prefill_ragged", "sc_decode_step_ragged", "sc_compress_ragged", "sc_cache_len_seq",
    "sc_schedule_rows", "sc_cache_reset_seq", "sc_cache_device_clock", "sc_steps_until_due",
    "sc_cache_note_replays",
    "sc_layers_workspace_bytes", "sc_layers_create", "sc_layers_get", "sc_layers_count", "sc_layers_destroy",
    "sc_layers_decode_step", "sc_layers_device_clock", "sc_layers_note_replays", "sc_layers_steps_until_due",
    "sc_layers_compress",
)


class sc_config(C.Structure):
    _fields_ = [(k, C.c_int32) for k in (
        "batch", "heads", "head_dim", "kv_dtype", "budget", "recent", "history", "drop",
        "trigger", "thresh_mode", "window_mode", "record_mode")] + [("scale", C.c_float)]


class ScError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (sc_status %d)" % (where, sc_status_str(status), status))


_lib = None


def lib():
    """Load ``libsc.so`` (built by ``__graft_entry__.build()`` / ``build.py``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libsc.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(hipcc --offload-arch=gfx950); there is no fallback implementation")
    l = C.CDLL(LIB_PATH)
    vp, i32p, i64p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    cfgp = C.POINTER(sc_config)
    l.sc_config_sizes.argtypes = [cfgp, i32p, i32p, i32p, i32p]
    l.sc_workspace_bytes.argtypes = [cfgp]
    l.sc_workspace_bytes.restype = C.c_size_t
    l.sc_schedule.argtypes = [cfgp, C.c_int64, i64p, i32p, i32p]
    l.sc_cache_create.argtypes = [cfgp, vp, C.c_size_t, vp, C.POINTER(vp)]
    l.sc_cache_reset.argtypes = [vp, vp]
    l.sc_cache_destroy.argtypes = [vp]
    l.sc_cache_destroy.restype = None
    l.sc_decode_step.argtypes = [vp, vp, vp, vp, C.c_int64, vp, vp, i32p, vp]
    l.sc_compress.argtypes = [vp, vp, vp, vp]
    l.sc_compress_static.argtypes = [vp, vp, vp, vp]
    l.sc_prefill.argtypes = [vp, vp, vp, vp, C.c_int32, C.c_int64, vp, vp, C.c_int32, vp]
    l.sc_prefill_plan.argtypes = [cfgp, C.c_int32, C.c_int32, C.c_int32, i32p, i32p, i32p, i32p]
    l.sc_cache_len.argtypes = [vp, i32p, i64p]
    l.sc_cache_view.argtypes = [vp] + [C.POINTER(vp)] * 6 + [i32p, i32p]
    l.sc_diag_persistence.argtypes = [vp, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_int32, vp, vp]
    l.sc_diag_kept_mass.argtypes = [vp, vp, C.c_int64, vp, vp]
    l.sc_diag_trace.argtypes = [vp, vp]
    l.sc_diag_read_bandwidth.argtypes = [vp, C.c_size_t, C.c_int32, vp, vp]
    l.sc_prefill_ragged.argtypes = [vp, vp, vp, vp, i32p, C.c_int64, vp, vp, C.c_int32, vp]
    l.sc_decode_step_ragged.argtypes = [vp, vp, vp, vp, C.c_int64, vp, vp, C.POINTER(C.c_uint8), i32p, vp]
    l.sc_compress_ragged.argtypes = [vp, vp, vp, vp]
    l.sc_cache_len_seq.argtypes = [vp, C.c_int32, i32p, i64p]
    l.sc_schedule_rows.argtypes = [cfgp, C.c_int64, i32p, i32p]
    l.sc_cache_reset_seq.argtypes = [vp, C.c_int32, vp]
    l.sc_cache_device_clock.argtypes = [vp, C.c_int32]
    l.sc_steps_until_due.argtypes = [vp, C.POINTER(C.c_uint8), i32p]
    l.sc_cache_note_replays.argtypes = [vp, C.c_int32, i32p]
    l.sc_layers_workspace_bytes.argtypes = [cfgp, C.c_int32, i32p, i32p]
    l.sc_layers_workspace_bytes.restype = C.c_size_t
    l.sc_layers_create.argtypes = [cfgp, C.c_int32, i32p, i32p, vp, C.c_size_t, vp, C.POINTER(vp)]
    l.sc_layers_get.argtypes = [vp, C.c_int32]
    l.sc_layers_get.restype = vp
    l.sc_layers_count.argtypes = [vp]
    l.sc_layers_count.restype = C.c_int32
    l.sc_layers_destroy.argtypes = [vp]
    l.sc_layers_destroy.restype = None
    l.sc_layers_decode_step.argtypes = [vp, vp, vp, vp, C.c_int64, C.c_int64, vp, C.c_int64, C.POINTER(C.c_uint8),
                                        i32p, vp]
    l.sc_layers_device_clock.argtypes = [vp, C.c_int32]
    l.sc_layers_note_replays.argtypes = [vp, C.c_int32, i32p]
    l.sc_layers_steps_until_due.argtypes = [vp, C.POINTER(C.c_uint8), i32p]
    l.sc_layers_compress.argtypes = [vp, i32p, vp]
    l.sc_status_str.argtypes = [C.c_int]
    l.sc_status_str.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("sc_workspace_bytes", "sc_cache_destroy", "sc_status_str", "sc_layers_workspace_bytes",
                        "sc_layers_get", "sc_layers_count", "sc_layers_destroy"):
            getattr(l, name).restype = C.c_int
    _lib = l
    return l


def _check(status: int, where: str):
    if status != SC_OK:
        raise ScError(status, where)


def make_config(batch, heads, head_dim, kv_dtype, budget, recent, history, drop,
                trigger=SC_TRIGGER_HARD_CAP, thresh_mode=SC_THRESH_INV_POS, scale=0.0,
                window_mode=SC_WINDOW_AUTO, record_mode=SC_RECORD_ONLINE) -> sc_config:
    return sc_config(batch, heads, head_dim, kv_dtype, budget, recent, history, drop, trigger,
                     thresh_mode, window_mode, record_mode, scale)


# ---- functions with the names of the C ABI -------------------------------------------------

def sc_status_str(status: int) -> str:
    return lib().sc_status_str(int(status)).decode()


def sc_config_sizes(cfg: sc_config):
    """-> (n_trig, capacity, buckets, ring_words)"""
    a, b, c, d = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib().sc_config_sizes(C.byref(cfg), C.byref(a), C.byref(b), C.byref(c), C.byref(d)),
           "sc_config_sizes")
    return a.value, b.value, c.value, d.value


def sc_workspace_bytes(cfg: sc_config) -> int:
    return int(lib().sc_workspace_bytes(C.byref(cfg)))


def sc_schedule(cfg: sc_config, t: int):
    """-> (epoch, bucket, counted)"""
    e, b, c = C.c_int64(), C.c_int32(), C.c_int32()
    _check(lib().sc_schedule(C.byref(cfg), int(t), C.byref(e), C.byref(b), C.byref(c)), "sc_schedule")
    return e.value, b.value, bool(c.value)


def sc_cache_create(cfg: sc_config, workspace_ptr: int, nbytes: int, stream: int = 0):
    h = C.c_void_p()
    _check(lib().sc_cache_create(C.byref(cfg), workspace_ptr, nbytes, stream, C.byref(h)),
           "sc_cache_create")
    return h


def sc_cache_reset(handle, stream=0) -> None:
    _check(lib().sc_cache_reset(handle, stream), "sc_cache_reset")


def sc_cache_destroy(handle) -> None:
    lib().sc_cache_destroy(handle)


def sc_decode_step(handle, q_ptr, k_ptr, v_ptr, in_stride, out_ptr, probs_ptr=None, stream=0) -> bool:
    """-> compress_due"""
    due = C.c_int32(0)
    _check(lib().sc_decode_step(handle, q_ptr, k_ptr, v_ptr, int(in_stride), out_ptr, probs_ptr,
                                C.byref(due), stream), "sc_decode_step")
    return bool(due.value)


def sc_compress(handle, evicted_ptr=None, probs_ptr=None, stream=0) -> None:
    _check(lib().sc_compress(handle, evicted_ptr, probs_ptr, stream), "sc_compress")


def sc_compress_static(handle, evicted_ptr=None, probs_ptr=None, stream=0) -> None:
    _check(lib().sc_compress_static(handle, evicted_ptr, probs_ptr, stream), "sc_compress_static")


def sc_prefill(handle, q_ptr, k_ptr, v_ptr, prompt_len, unit_stride, out_ptr=None, probs_ptr=None,
               mode=SC_PREFILL_AUTO, stream=0) -> None:
    _check(lib().sc_prefill(handle, q_ptr, k_ptr, v_ptr, int(prompt_len), int(unit_stride), out_ptr,
                            probs_ptr, int(mode), stream), "sc_prefill")


def sc_prefill_plan(cfg: sc_config, prompt_len: int, mode: int = SC_PREFILL_AUTO):
    """-> list of (run_len, dense, compress_follows)"""
    n = C.c_int32()
    _check(lib().sc_prefill_plan(C.byref(cfg), prompt_len, mode, 0, None, None, None, C.byref(n)),
           "sc_prefill_plan")
    arr = [(C.c_int32 * n.value)() for _ in range(3)]
    _check(lib().sc_prefill_plan(C.byref(cfg), prompt_len, mode, n.value, arr[0], arr[1], arr[2],
                                 C.byref(n)), "sc_prefill_plan")
    return [(arr[0][i], bool(arr[1][i]), bool(arr[2][i])) for i in range(n.value)]


def sc_cache_len(handle):
    """-> (n, t)"""
    n, t = C.c_int32(), C.c_int64()
    _check(lib().sc_cache_len(handle, C.byref(n), C.byref(t)), "sc_cache_len")
    return n.value, t.value


def sc_schedule_rows(cfg: sc_config, t: int):
    """-> (rows right after step t, compression due after it)"""
    n, due = C.c_int32(), C.c_int32()
    _check(lib().sc_schedule_rows(C.byref(cfg), int(t), C.byref(n), C.byref(due)), "sc_schedule_rows")
    return n.value, bool(due.value)


def sc_cache_reset_seq(handle, b: int, stream=0) -> None:
    _check(lib().sc_cache_reset_seq(handle, int(b), stream), "sc_cache_reset_seq")


def sc_cache_len_seq(handle, b: int):
    """-> (n_b, t_b)"""
    n, t = C.c_int32(), C.c_int64()
    _check(lib().sc_cache_len_seq(handle, int(b), C.byref(n), C.byref(t)), "sc_cache_len_seq")
    return n.value, t.value


def sc_prefill_ragged(handle, q_ptr, k_ptr, v_ptr, prompt_len, unit_stride, out_ptr=None, probs_ptr=None,
                      mode=SC_PREFILL_AUTO, stream=0) -> None:
    """prompt_len: one length per sequence (0 = leave the sequence alone)."""
    arr = (C.c_int32 * len(prompt_len))(*[int(x) for x in prompt_len])
    _check(lib().sc_prefill_ragged(handle, q_ptr, k_ptr, v_ptr, arr, int(unit_stride), out_ptr, probs_ptr,
                                   int(mode), stream), "sc_prefill_ragged")


def sc_decode_step_ragged(handle, q_ptr, k_ptr, v_ptr, in_stride, out_ptr, probs_ptr=None, active=None,
                          stream=0) -> int:
    """active: one flag per sequence or None (all).  -> number of sequences now due."""
    arr = None if active is None else (C.c_uint8 * len(active))(*[1 if x else 0 for x in active])
    due = C.c_int32(0)
    _check(lib().sc_decode_step_ragged(handle, q_ptr, k_ptr, v_ptr, int(in_stride), out_ptr, probs_ptr, arr,
                                       C.byref(due), stream), "sc_decode_step_ragged")
    return due.value


def sc_compress_ragged(handle, evicted_ptr=None, probs_ptr=None, stream=0) -> None:
    _check(lib().sc_compress_ragged(handle, evicted_ptr, probs_ptr, stream), "sc_compress_ragged")


def sc_cache_view(handle):
    """-> dict of raw device addresses plus capacity and buckets"""
    ptrs = [C.c_void_p() for _ in range(6)]
    cap, bk = C.c_int32(), C.c_int32()
    _check(lib().sc_cache_view(handle, *[C.byref(p) for p in ptrs], C.byref(cap), C.byref(bk)),
           "sc_cache_view")
    names = ("K", "V", "K_meta", "V_meta", "pos", "cnt")
    d = {k: (p.value or 0) for k, p in zip(names, ptrs)}
    d["capacity"], d["buckets"] = cap.value, bk.value
    return d


def sc_diag_persistence(probs_ptr, units, length, row_stride, unit_stride, split, counts_ptr, stream=0) -> None:
    _check(lib().sc_diag_persistence(probs_ptr, units, length, int(row_stride), int(unit_stride), split,
                                     counts_ptr, stream), "sc_diag_persistence")


def sc_diag_kept_mass(handle, probs_full_ptr, unit_stride, mass_ptr, stream=0) -> None:
    _check(lib().sc_diag_kept_mass(handle, probs_full_ptr, int(unit_stride), mass_ptr, stream),
           "sc_diag_kept_mass")


def sc_diag_read_bandwidth(buf_ptr, nbytes: int, nontemporal: bool, sink_ptr, stream=0) -> None:
    _check(lib().sc_diag_read_bandwidth(buf_ptr, int(nbytes), 1 if nontemporal else 0, sink_ptr, stream),
           "sc_diag_read_bandwidth")


def sc_diag_trace(handle, trace_ptr=None) -> None:
    _check(lib().sc_diag_trace(handle, trace_ptr), "sc_diag_trace")


# ---- a small holder that keeps the torch workspace alive next to the handle ----------------

class BudgetCache:
    """Owns a torch uint8 workspace tensor and the ``sc_cache`` handle living in it.

    Marshalling only: every method forwards to the C entry point of the same name with the
    tensors' device addresses and the current torch stream."""

    def __init__(self, cfg: sc_config, device="cuda:0", _borrowed=None):
        """`_borrowed` = (handle, workspace tensor) of a cache owned by a LayerSet."""
        import torch

        self._torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        self.n_trig, self.capacity, self.buckets, self.ring_words = sc_config_sizes(cfg)
        self.units = cfg.batch * cfg.heads
        self.io_dtype = torch.float32 if cfg.kv_dtype == SC_KV_F32 else torch.float16
        if _borrowed is not None:
            self.handle, self.workspace = _borrowed
            self._destroy = lambda h: None
        else:
            nbytes = sc_workspace_bytes(cfg)
            self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
            base = self.workspace.data_ptr()
            self._ws_ptr = (base + 255) // 256 * 256
            self.handle = sc_cache_create(cfg, self._ws_ptr, nbytes, self._stream())
            self._destroy = lib().sc_cache_destroy  # kept here: module globals may be gone at interpreter exit
        self._view = sc_cache_view(self.handle)

    def _stream(self) -> int:
        return int(self._torch.cuda.current_stream(self.device).cuda_stream)

    def reset(self) -> None:
        sc_cache_reset(self.handle, self._stream())

    def close(self):
        if getattr(self, "handle", None):
            self._destroy(self.handle)
            self.handle = None

    __del__ = close

    @property
    def n(self):
        return sc_cache_len(self.handle)[0]

    @property
    def t(self):
        return sc_cache_len(self.handle)[1]

    def decode_step(self, q, k_new, v_new, out, probs_out=None, in_stride=0) -> bool:
        return sc_decode_step(self.handle, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), in_stride,
                              out.data_ptr(), None if probs_out is None else probs_out.data_ptr(),
                              self._stream())

    def compress(self, evicted_out=None, probs_out=None) -> None:
        sc_compress(self.handle, None if evicted_out is None else evicted_out.data_ptr(),
                    None if probs_out is None else probs_out.data_ptr(), self._stream())

    def compress_static(self, evicted_out=None, probs_out=None) -> None:
        sc_compress_static(self.handle, None if evicted_out is None else evicted_out.data_ptr(),
                           None if probs_out is None else probs_out.data_ptr(), self._stream())

    def prefill(self, q, k, v, prompt_len, unit_stride=0, out=None, probs_out=None,
                mode=SC_PREFILL_AUTO) -> None:
        sc_prefill(self.handle, q.data_ptr(), k.data_ptr(), v.data_ptr(), prompt_len, unit_stride,
                   None if out is None else out.data_ptr(),
                   None if probs_out is None else probs_out.data_ptr(), mode, self._stream())

    # -- ragged batches: every sequence on its own clock --
    def len_seq(self, b: int):
        return sc_cache_len_seq(self.handle, b)

    def reset_seq(self, b: int) -> None:
        sc_cache_reset_seq(self.handle, b, self._stream())

    def device_clock(self, enable: bool = True) -> None:
        _check(lib().sc_cache_device_clock(self.handle, 1 if enable else 0), "sc_cache_device_clock")

    def steps_until_due(self, active=None) -> int:
        arr = None if active is None else (C.c_uint8 * len(active))(*[1 if x else 0 for x in active])
        k = C.c_int32()
        _check(lib().sc_steps_until_due(self.handle, arr, C.byref(k)), "sc_steps_until_due")
        return k.value

    def note_replays(self, k: int = 1) -> int:
        due = C.c_int32()
        _check(lib().sc_cache_note_replays(self.handle, int(k), C.byref(due)), "sc_cache_note_replays")
        return due.value

    def prefill_ragged(self, q, k, v, prompt_len, unit_stride=0, out=None, probs_out=None,
                       mode=SC_PREFILL_AUTO) -> None:
        sc_prefill_ragged(self.handle, q.data_ptr(), k.data_ptr(), v.data_ptr(), prompt_len, unit_stride,
                          None if out is None else out.data_ptr(),
                          None if probs_out is None else probs_out.data_ptr(), mode, self._stream())

    def decode_step_ragged(self, q, k_new, v_new, out, probs_out=None, in_stride=0, active=None) -> int:
        return sc_decode_step_ragged(self.handle, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), in_stride,
                                     out.data_ptr(), None if probs_out is None else probs_out.data_ptr(),
                                     active, self._stream())

    def compress_ragged(self, evicted_out=None, probs_out=None) -> None:
        sc_compress_ragged(self.handle, None if evicted_out is None else evicted_out.data_ptr(),
                           None if probs_out is None else probs_out.data_ptr(), self._stream())

    def _typed(self, key, dtype, shape):
        """A torch view (no copy) of one of the cache's arrays inside the workspace."""
        torch = self._torch
        off = self._view[key] - self.workspace.data_ptr()
        nbytes = int(torch.tensor([], dtype=dtype).element_size())
        count = 1
        for s in shape:
            count *= s
        return self.workspace[off: off + count * nbytes].view(dtype).view(*shape)

    def pos(self):
        return self._typed("pos", self._torch.int32, (self.units, self.capacity))

    def cnt(self):
        """Bucket mode: int16 view [U, buckets, C] of the 16-bit counters (empty in ring mode)."""
        return self._typed("cnt", self._torch.int16, (self.units, self.buckets, self.capacity))

    def ring(self):
        """Ring mode: int32 view [U, ring_words, C] of the per-slot rings (empty in bucket mode)."""
        return self._typed("cnt", self._torch.int32, (self.units, self.ring_words, self.capacity))

    def kv_rows(self):
        """(K, V) as stored: F32/F16 -> [U, C, d] tensors; I4G64 -> uint8 codes [U, C, d/2]."""
        torch = self._torch
        d = self.cfg.head_dim
        if self.cfg.kv_dtype == SC_KV_I4G64:
            shape, dt = (self.units, self.capacity, d // 2), torch.uint8
        else:
            shape, dt = (self.units, self.capacity, d), self.io_dtype
        return self._typed("K", dt, shape), self._typed("V", dt, shape)

    def kv_meta(self):
        """I4G64 only: (K_meta, V_meta) as fp16 [U, C, d/64, 2] = (scale, zero)."""
        torch = self._torch
        shape = (self.units, self.capacity, self.cfg.head_dim // 64, 2)
        return self._typed("K_meta", torch.float16, shape), self._typed("V_meta", torch.float16, shape)


def kv_cache_bytes(layers: int, d_model: int, batch: int, seq: int, bytes_per_elem: int = 2) -> int:
    """Bytes of a full (uncompressed) KV cache: two tensors of [batch, seq, d_model] per layer
    (the accounting behind the memory table of the paper's introduction)."""
    return 2 * layers * d_model * bytes_per_elem * batch * seq


class LayerSet:
    """One cache per layer with per-layer budgets, in one torch workspace (sc_layers_*)."""

    def __init__(self, cfg: sc_config, budgets, drops=None, device="cuda:0"):
        import copy

        import torch

        self.device = torch.device(device)
        L = len(budgets)
        b = (C.c_int32 * L)(*[int(x) for x in budgets])
        m = None if drops is None else (C.c_int32 * L)(*[int(x) for x in drops])
        nbytes = int(lib().sc_layers_workspace_bytes(C.byref(cfg), L, b, m))
        if nbytes == 0:
            raise ScError(SC_ERR_INVALID_ARG, "sc_layers_workspace_bytes")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        ws = (self.workspace.data_ptr() + 255) // 256 * 256
        h = C.c_void_p()
        stream = int(torch.cuda.current_stream(self.device).cuda_stream)
        _check(lib().sc_layers_create(C.byref(cfg), L, b, m, ws, nbytes, stream, C.byref(h)), "sc_layers_create")
        self.handle = h
        self._destroy = lib().sc_layers_destroy
        self.layers = []
        for l in range(L):
            c = copy.copy(cfg)
            c.budget = int(budgets[l])
            if drops is not None:
                c.drop = int(drops[l])
            self.layers.append(BudgetCache(c, device, _borrowed=(C.c_void_p(lib().sc_layers_get(h, l)),
                                                                 self.workspace)))
        assert lib().sc_layers_count(h) == L

    def __len__(self):
        return len(self.layers)

    def _stream(self) -> int:
        import torch
        return int(torch.cuda.current_stream(self.device).cuda_stream)

    def decode_step(self, q, k_new, v_new, out, in_stride=0, active=None) -> int:
        """q, k_new, v_new, out: [L, U, d] tensors (a layer's block may be strided).  -> pairs now due."""
        arr = None if active is None else (C.c_uint8 * len(active))(*[1 if x else 0 for x in active])
        due = C.c_int32(0)
        _check(lib().sc_layers_decode_step(self.handle, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                           q.stride(0), in_stride, out.data_ptr(), out.stride(0), arr,
                                           C.byref(due), self._stream()), "sc_layers_decode_step")
        return due.value

    def device_clock(self, enable: bool = True) -> None:
        _check(lib().sc_layers_device_clock(self.handle, 1 if enable else 0), "sc_layers_device_clock")

    def note_replays(self, k: int = 1) -> int:
        due = C.c_int32(0)
        _check(lib().sc_layers_note_replays(self.handle, int(k), C.byref(due)), "sc_layers_note_replays")
        return due.value

    def steps_until_due(self, active=None) -> int:
        arr = None if active is None else (C.c_uint8 * len(active))(*[1 if x else 0 for x in active])
        k = C.c_int32()
        _check(lib().sc_layers_steps_until_due(self.handle, arr, C.byref(k)), "sc_layers_steps_until_due")
        return k.value

    def compress(self) -> int:
        n = C.c_int32(0)
        _check(lib().sc_layers_compress(self.handle, C.byref(n), self._stream()), "sc_layers_compress")
        return n.value

    def __getitem__(self, l):
        return self.layers[l]

    def close(self):
        if getattr(self, "handle", None):
            for c in self.layers:
                c.handle = None
            self._destroy(self.handle)
            self.handle = None

    __del__ = close
