"""ctypes binding of libodma: argument marshalling only.

Every function here has the name and the argument order of the C entry point it
calls (include/odma.h).  Host arrays are numpy arrays; DEVICE arguments are
torch CUDA tensors (or raw integer addresses) whose ``data_ptr()`` is passed
through.  There is no fallback: if the shared library has not been built the
import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ODMA_LIB") or os.path.join(_HERE, "libodma.so")   # ODMA_LIB: load another build of the library

OK, INVALID_ARG, NOMEM, OVERFLOW, UNKNOWN_REQ, HIP_ERROR = 0, -1, -2, -3, -4, -5
F32, BF16, FP8 = 0, 1, 2
ARENA_MAIN, ARENA_SAFETY = 0, 1
BLOCK_TOKENS = 16
KERNEL_AUTO, KERNEL_VALU, KERNEL_MFMA = 0, 1, 2
REUSE_PLAN, SKIP_REDUCE = 1, 2
MIGRATE_DEFER_RELEASE = 1
TUNE_WAVES_PER_CU, TUNE_ITEMS_PER_WAVE, TUNE_MIN_CHUNK, TUNE_PIPELINE_DEPTH, TUNE_WAVES_PER_WG = 1, 2, 3, 4, 5
TUNE_ODD_XCD_WEIGHT = 6
TUNE_LATE_WAVE_WEIGHT = 7
TUNE_FUSE_REDUCE = 8
TUNE_PREFILL_COLUMN_TILES = 9

EXPORTS = [
    "odma_workspace_bytes", "odma_pool_create", "odma_pool_destroy", "odma_inflate", "odma_assign",
    "odma_release", "odma_advance", "odma_migrate", "odma_recalibrate", "odma_pool_snapshot",
    "odma_pool_free_extents", "odma_pool_stats", "odma_pool_lookup", "odma_append_kv",
    "odma_decode_attention", "odma_gather_kv", "odma_pool_decode_kernel", "odma_last_error", "odma_version",
    "odma_pool_tune", "odma_decode_step", "odma_stream_read_probe", "odma_recalibrator_start",
    "odma_report_completions", "odma_recalibrator_drain", "odma_recalibrator_stop", "odma_migrate_batch",
    "odma_migrate_finish", "odma_prefill_attention", "odma_block_read_probe", "odma_stream_plan_ranges",
    "odma_decode_attention_static",
]


class OdmaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libodma error {code}: {msg}")
        self.code = code


class odma_pool_config_t(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("kv_dtype", C.c_int32), ("out_dtype", C.c_int32), ("align_tokens", C.c_int32), ("large_cap", C.c_int32),
        ("main_tokens", C.c_int64), ("safety_tokens", C.c_int64),
        ("max_requests", C.c_int32), ("n_buckets", C.c_int32),
        ("boundaries", C.POINTER(C.c_int32)), ("quantile_num", C.POINTER(C.c_int32)),
        ("quantile_den", C.POINTER(C.c_int32)),
        ("window", C.c_int32), ("decode_kernel", C.c_int32),
        ("gamma", C.c_double), ("tau", C.c_double),
        ("sm_scale", C.c_float), ("max_splits", C.c_int32),
        ("k_scale", C.c_float), ("v_scale", C.c_float),
        ("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
    ]


class odma_pool_stats_t(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "live_requests", "live_tokens", "live_reserved", "main_free", "safety_free", "done_requests",
        "done_actual", "done_reserved", "done_reserved_both", "migrations", "nomem", "recalibrations",
        "boundary_epoch")]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_09427_amd.build` "
                          "(there is no CPU fallback)")
    # Device pointers and streams come from PyTorch, so the library must run on PyTorch's HIP runtime.
    # PyTorch ships its own copy of that runtime; with it in the process first, the loader binds the
    # library's dependency to that copy.  Loaded the other way round the process ends up with two
    # runtimes and the second one finds no device.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    i32p, i64p, f32p, vp = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_float), C.c_void_p
    cfgp = C.POINTER(odma_pool_config_t)
    sig = {
        "odma_workspace_bytes": (C.c_size_t, [cfgp]),
        "odma_pool_create": (C.c_int, [cfgp, C.POINTER(vp)]),
        "odma_pool_destroy": (C.c_int, [vp]),
        "odma_inflate": (C.c_int64, [vp, C.c_int32, C.c_float]),
        "odma_assign": (C.c_int, [vp, C.c_int32, i32p, i32p, f32p, i32p, i32p, C.c_int32, i32p, i64p, i32p, i32p]),
        "odma_release": (C.c_int, [vp, C.c_int32, i32p, i32p]),
        "odma_advance": (C.c_int, [vp, C.c_int32, i32p, i32p, i32p, i32p]),
        "odma_migrate": (C.c_int, [vp, C.c_int32, vp, i64p, i32p]),
        "odma_recalibrate": (C.c_int, [vp, C.c_int32, i32p, i32p]),
        "odma_pool_snapshot": (C.c_int, [vp, C.c_int32, i32p, i32p, i32p, i64p, i32p, i32p, i32p]),
        "odma_pool_free_extents": (C.c_int, [vp, C.c_int32, C.c_int32, i32p, i64p, i64p]),
        "odma_pool_stats": (C.c_int, [vp, C.POINTER(odma_pool_stats_t)]),
        "odma_pool_lookup": (C.c_int, [vp, C.c_int32, i32p, i64p, i32p, i32p]),
        "odma_append_kv": (C.c_int, [vp, C.c_int32, C.c_int32, vp, vp, vp, vp, C.c_int32, vp, C.c_int32, vp, vp, vp]),
        "odma_decode_attention": (C.c_int, [vp, C.c_int32, C.c_int32, vp, vp, vp, vp, C.c_int32, vp, C.c_uint32, vp]),
        "odma_decode_attention_static": (C.c_int, [vp, C.c_int32, C.c_int32, vp, vp, vp, vp, C.c_int32, vp, C.c_uint32, vp]),
        "odma_stream_plan_ranges": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, i32p, i32p]),
        "odma_prefill_attention": (C.c_int, [vp, C.c_int32, C.c_int32, vp, C.c_int64, vp, vp, vp, vp, vp, C.c_int32, vp, vp]),
        "odma_decode_step": (C.c_int, [vp, C.c_int32, C.c_int32, vp, vp, vp, vp, vp, vp, C.c_int32, vp, C.c_uint32, vp]),
        "odma_gather_kv": (C.c_int, [vp, C.c_int32, C.c_int64, C.c_int32, vp, vp, vp, vp]),
        "odma_stream_read_probe": (C.c_int, [vp, C.c_size_t, vp, vp]),
        "odma_block_read_probe": (C.c_int, [vp, vp, vp, C.c_int64, vp, vp]),
        "odma_migrate_batch": (C.c_int, [vp, C.c_int32, i32p, C.c_uint32, vp, i64p, i32p, i32p]),
        "odma_migrate_finish": (C.c_int, [vp, C.c_int32, i32p, i32p]),
        "odma_recalibrator_start": (C.c_int, [vp, C.c_int32]),
        "odma_report_completions": (C.c_int, [vp, C.c_int32, i32p]),
        "odma_recalibrator_drain": (C.c_int, [vp, i64p]),
        "odma_recalibrator_stop": (C.c_int, [vp]),
        "odma_pool_decode_kernel": (C.c_int, [vp]),
        "odma_pool_tune": (C.c_int, [vp, C.c_int32, C.c_int32]),
        "odma_last_error": (C.c_char_p, []),
        "odma_version": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


lib = _load()


# ---- marshalling helpers -------------------------------------------------------------

def _i32(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray], ctype):
    return None if a is None else a.ctypes.data_as(C.POINTER(ctype))


def _dev(t) -> Optional[int]:
    """Device address of a torch tensor (must be contiguous) or a raw integer address."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise TypeError("DEVICE argument must be a CUDA tensor")
    if not t.is_contiguous():
        raise ValueError("DEVICE argument must be contiguous")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def odma_last_error() -> str:
    return lib.odma_last_error().decode()


def odma_version() -> str:
    return lib.odma_version().decode()


def odma_stream_read_probe(buf, n_bytes: int, sink, stream=None):
    return _check(lib.odma_stream_read_probe(_dev(buf), int(n_bytes), _dev(sink), _stream(stream)))


def odma_block_read_probe(k_plane, v_plane, table, n_steps: int, sink, stream=None):
    return _check(lib.odma_block_read_probe(_dev(k_plane), _dev(v_plane), _dev(table), int(n_steps), _dev(sink),
                                            _stream(stream)))


def odma_stream_plan_ranges(total_tiles: int, n_waves: int, waves_per_wg: int = 4, min_tiles: int = 4,
                            odd_xcd_weight: int = 256, late_wave_weight: int = 256):
    """Returns (start[n_waves + 1], waves_used)."""
    start = np.zeros(n_waves + 1, np.int32)
    used = C.c_int32(0)
    _check(lib.odma_stream_plan_ranges(int(total_tiles), int(n_waves), int(waves_per_wg), int(min_tiles),
                                       int(odd_xcd_weight), int(late_wave_weight), _ptr(start, C.c_int32), C.byref(used)))
    return start, used.value


def _check(rc: int, allow: Sequence[int] = ()):
    if rc != OK and rc not in allow:
        raise OdmaError(rc, odma_last_error())
    return rc


# ---- configuration ----------------------------------------------------------------------

def make_config(*, n_layers, n_q_heads, n_kv_heads, head_dim, kv_dtype, out_dtype, main_tokens, safety_tokens,
                large_cap, boundaries, max_requests, align_tokens=16, quantiles=None, window=10000,
                decode_kernel=KERNEL_AUTO, gamma=0.2, tau=0.8, sm_scale=0.0, max_splits=0, k_scale=0.0, v_scale=0.0,
                k_pool=None, v_pool=None, workspace=None):
    """Fills an odma_pool_config_t.  Returns (cfg, keepalive): the arrays cfg points at."""
    cfg = odma_pool_config_t()
    b = _i32(list(boundaries))
    keep = [b]
    cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim = n_layers, n_q_heads, n_kv_heads, head_dim
    cfg.kv_dtype, cfg.out_dtype, cfg.align_tokens, cfg.large_cap = kv_dtype, out_dtype, align_tokens, large_cap
    cfg.main_tokens, cfg.safety_tokens = main_tokens, safety_tokens
    cfg.max_requests, cfg.n_buckets = max_requests, len(b)
    cfg.boundaries = _ptr(b, C.c_int32)
    if quantiles is not None:
        qn, qd = _i32([q[0] for q in quantiles]), _i32([q[1] for q in quantiles])
        keep += [qn, qd]
        cfg.quantile_num, cfg.quantile_den = _ptr(qn, C.c_int32), _ptr(qd, C.c_int32)
    cfg.window, cfg.decode_kernel = window, decode_kernel
    cfg.gamma, cfg.tau, cfg.sm_scale, cfg.max_splits = gamma, tau, sm_scale, max_splits
    cfg.k_scale, cfg.v_scale = k_scale, v_scale
    cfg.k_pool, cfg.v_pool, cfg.workspace = _dev(k_pool), _dev(v_pool), _dev(workspace)
    cfg.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    keep += [k_pool, v_pool, workspace]
    return cfg, keep


def odma_workspace_bytes(cfg: odma_pool_config_t) -> int:
    n = lib.odma_workspace_bytes(C.byref(cfg))
    if n == 0:
        raise OdmaError(INVALID_ARG, odma_last_error())
    return n


# ---- the pool -----------------------------------------------------------------------------

class Pool:
    """Owns one odma_pool_t.  Methods are named after the C calls they make."""

    def __init__(self, cfg: odma_pool_config_t, keepalive=None):
        self._keep = keepalive
        self.cfg = cfg
        h = C.c_void_p()
        _check(lib.odma_pool_create(C.byref(cfg), C.byref(h)))
        self._h = h
        self._destroy = lib.odma_pool_destroy            # kept: module globals may be gone when __del__ runs at exit
        self.n_buckets = cfg.n_buckets

    def close(self):
        if getattr(self, "_h", None):
            self._destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    # -- host ------------------------------------------------------------------------
    def odma_inflate(self, pred_len: int, u: float) -> int:
        return lib.odma_inflate(self._h, int(pred_len), float(u))

    def odma_assign(self, req_id, pred_len, uncertainty=None, prompt_len=None, boundaries=None):
        """Returns (rc, bucket, offset, cap, status); rc is the first per-request error."""
        rid, pl = _i32(req_id), _i32(pred_len)
        n = len(rid)
        u = None if uncertainty is None else np.ascontiguousarray(uncertainty, dtype=np.float32)
        pr, b = _i32(prompt_len), _i32(boundaries)
        bucket, cap, status = (np.zeros(n, np.int32) for _ in range(3))
        offset = np.zeros(n, np.int64)
        rc = lib.odma_assign(self._h, n, _ptr(rid, C.c_int32), _ptr(pl, C.c_int32), _ptr(u, C.c_float),
                             _ptr(pr, C.c_int32), _ptr(b, C.c_int32), 0 if b is None else len(b),
                             _ptr(bucket, C.c_int32), _ptr(offset, C.c_int64), _ptr(cap, C.c_int32),
                             _ptr(status, C.c_int32))
        return rc, bucket, offset, cap, status

    def odma_release(self, req_id):
        rid = _i32(req_id)
        status = np.zeros(len(rid), np.int32)
        rc = lib.odma_release(self._h, len(rid), _ptr(rid, C.c_int32), _ptr(status, C.c_int32))
        return rc, status

    def odma_advance(self, req_id, n_new=None):
        rid, nn = _i32(req_id), _i32(n_new)
        overflow, status = np.zeros(len(rid), np.int32), np.zeros(len(rid), np.int32)
        rc = lib.odma_advance(self._h, len(rid), _ptr(rid, C.c_int32), _ptr(nn, C.c_int32),
                              _ptr(overflow, C.c_int32), _ptr(status, C.c_int32))
        return rc, overflow, status

    def odma_migrate(self, req_id: int, stream=None):
        """Returns (rc, new_offset, new_cap)."""
        off, cap = C.c_int64(-1), C.c_int32(0)
        has_dev = bool(self.cfg.k_pool)
        rc = lib.odma_migrate(self._h, int(req_id), _stream(stream) if has_dev else None, C.byref(off), C.byref(cap))
        return rc, off.value, cap.value

    def odma_migrate_batch(self, req_id, flags: int = 0, stream=None):
        """Returns (rc, new_offset[], new_cap[], status[])."""
        rid = _i32(req_id)
        n = len(rid)
        off, cap, st = np.full(n, -1, np.int64), np.zeros(n, np.int32), np.zeros(n, np.int32)
        has_dev = bool(self.cfg.k_pool)
        rc = lib.odma_migrate_batch(self._h, n, _ptr(rid, C.c_int32), flags, _stream(stream) if has_dev else None,
                                    _ptr(off, C.c_int64), _ptr(cap, C.c_int32), _ptr(st, C.c_int32))
        return rc, off, cap, st

    def odma_migrate_finish(self, req_id):
        """Returns (rc, status[])."""
        rid = _i32(req_id)
        st = np.zeros(len(rid), np.int32)
        rc = lib.odma_migrate_finish(self._h, len(rid), _ptr(rid, C.c_int32), _ptr(st, C.c_int32))
        return rc, st

    def odma_recalibrate(self, realized_len=()):
        rl = _i32(list(realized_len))
        out = np.zeros(self.n_buckets, np.int32)
        _check(lib.odma_recalibrate(self._h, len(rl), _ptr(rl, C.c_int32), _ptr(out, C.c_int32)))
        return tuple(int(x) for x in out)

    def odma_recalibrator_start(self, refresh_every: int):
        return _check(lib.odma_recalibrator_start(self._h, int(refresh_every)))

    def odma_report_completions(self, realized_len):
        rl = _i32(list(realized_len))
        return _check(lib.odma_report_completions(self._h, len(rl), _ptr(rl, C.c_int32)))

    def odma_recalibrator_drain(self) -> int:
        epoch = C.c_int64(0)
        _check(lib.odma_recalibrator_drain(self._h, C.byref(epoch)))
        return epoch.value

    def odma_recalibrator_stop(self):
        return _check(lib.odma_recalibrator_stop(self._h))

    def odma_pool_snapshot(self):
        """Returns (list of (id, arena, offset, cap, len), boundaries)."""
        n = C.c_int32(0)
        b = np.zeros(self.n_buckets, np.int32)
        _check(lib.odma_pool_snapshot(self._h, 0, C.byref(n), None, None, None, None, None, _ptr(b, C.c_int32)))
        k = n.value
        rid, arena, cap, ln = (np.zeros(k, np.int32) for _ in range(4))
        off = np.zeros(k, np.int64)
        _check(lib.odma_pool_snapshot(self._h, k, C.byref(n), _ptr(rid, C.c_int32), _ptr(arena, C.c_int32),
                                      _ptr(off, C.c_int64), _ptr(cap, C.c_int32), _ptr(ln, C.c_int32), None))
        rows = [(int(rid[i]), int(arena[i]), int(off[i]), int(cap[i]), int(ln[i])) for i in range(k)]
        return rows, tuple(int(x) for x in b)

    def odma_pool_free_extents(self, arena: int):
        n = C.c_int32(0)
        _check(lib.odma_pool_free_extents(self._h, arena, 0, C.byref(n), None, None))
        k = n.value
        start, size = np.zeros(k, np.int64), np.zeros(k, np.int64)
        _check(lib.odma_pool_free_extents(self._h, arena, k, C.byref(n), _ptr(start, C.c_int64), _ptr(size, C.c_int64)))
        return [(int(start[i]), int(size[i])) for i in range(k)]

    def odma_pool_stats(self) -> dict:
        s = odma_pool_stats_t()
        _check(lib.odma_pool_stats(self._h, C.byref(s)))
        return {name: getattr(s, name) for name, _ in odma_pool_stats_t._fields_}

    def odma_pool_lookup(self, req_id):
        rid = _i32(req_id)
        n = len(rid)
        off, ln, cap = np.zeros(n, np.int64), np.zeros(n, np.int32), np.zeros(n, np.int32)
        _check(lib.odma_pool_lookup(self._h, n, _ptr(rid, C.c_int32), _ptr(off, C.c_int64), _ptr(ln, C.c_int32),
                                    _ptr(cap, C.c_int32)))
        return off, ln, cap

    def odma_pool_decode_kernel(self) -> int:
        return lib.odma_pool_decode_kernel(self._h)

    def odma_pool_tune(self, knob: int, value: int):
        return _check(lib.odma_pool_tune(self._h, knob, value))

    # -- device ------------------------------------------------------------------------
    def odma_append_kv(self, layer, n, offsets, positions, n_new, src_start, max_new, block_table, bt_stride,
                       k_new, v_new, stream=None):
        _check(lib.odma_append_kv(self._h, layer, n, _dev(offsets), _dev(positions), _dev(n_new), _dev(src_start),
                                  max_new, _dev(block_table), bt_stride, _dev(k_new), _dev(v_new), _stream(stream)))

    def odma_decode_attention(self, layer, n, q, offsets, lengths, block_table, bt_stride, out, flags=0, stream=None):
        _check(lib.odma_decode_attention(self._h, layer, n, _dev(q), _dev(offsets), _dev(lengths), _dev(block_table),
                                         bt_stride, _dev(out), flags, _stream(stream)))

    def odma_decode_attention_static(self, layer, n, q, offsets, lengths, block_table, bt_stride, out, flags=0,
                                     stream=None):
        _check(lib.odma_decode_attention_static(self._h, layer, n, _dev(q), _dev(offsets), _dev(lengths),
                                                _dev(block_table), bt_stride, _dev(out), flags, _stream(stream)))

    def odma_decode_step(self, layer, n, q, k_new, v_new, offsets, lengths, block_table, bt_stride, out, flags=0,
                         stream=None):
        _check(lib.odma_decode_step(self._h, layer, n, _dev(q), _dev(k_new), _dev(v_new), _dev(offsets), _dev(lengths),
                                    _dev(block_table), bt_stride, _dev(out), flags, _stream(stream)))

    def odma_prefill_attention(self, layer, n, q, total_q, q_start, n_q, offsets, lengths, block_table, bt_stride, out,
                               stream=None):
        _check(lib.odma_prefill_attention(self._h, layer, n, _dev(q), int(total_q), _dev(q_start), _dev(n_q), _dev(offsets),
                                          _dev(lengths), _dev(block_table), bt_stride, _dev(out), _stream(stream)))

    def odma_gather_kv(self, layer, offset, length, block_row, k_out, v_out, stream=None):
        _check(lib.odma_gather_kv(self._h, layer, int(offset), int(length), _dev(block_row), _dev(k_out), _dev(v_out),
                                  _stream(stream)))
