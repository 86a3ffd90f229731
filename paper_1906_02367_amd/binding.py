"""Python face of the C-ABI library `libqsl.so` (see include/qsl.h): argument marshalling only.

Every step of the hot path runs in the HIP kernels behind the C ABI; torch is used for device
memory and for the current HIP stream.  Importing this module loads the library and raises if
it has not been built -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

from .build import LIB_PATH

TOPK, RANDK = 0, 1
QSGD, SIGN_L1, SIGN_L2, FP32, QSGD_SCALED, SIGN_L3, SIGN_L4 = 0, 1, 2, 3, 4, 5, 6
FLAG_NO_FAST_PATH = 1
FLAG_NO_SMALL_PATH = 2
FLAG_OWN_V = 4
FLAG_NO_WARM_START = 8
FLAG_DENSE_FORMAT = 16

OK, ERR_INVALID_ARG, ERR_BUFFER_TOO_SMALL, ERR_NONFINITE_INPUT, ERR_DEVICE, ERR_UNSUPPORTED = range(6)


class QslError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {_lib.qsl_status_string(status).decode()} (status {int(status)})")


class _Config(C.Structure):
    _fields_ = [("d", C.c_uint64), ("num_segments", C.c_uint32), ("seg_offset", C.POINTER(C.c_uint64)),
                ("seg_k", C.POINTER(C.c_uint32)), ("s", C.c_uint32), ("sparsifier", C.c_uint32),
                ("quantizer", C.c_uint32), ("seed", C.c_uint64), ("max_workers", C.c_uint32), ("flags", C.c_uint32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_1906_02367_amd.build, or "
                          f"__graft_entry__.build()); this package has no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, u32, u64 = C.c_void_p, C.c_uint32, C.c_uint64
    lib.qsl_status_string.argtypes = [C.c_int]; lib.qsl_status_string.restype = C.c_char_p
    lib.qsl_create.argtypes = [C.POINTER(vp), C.POINTER(_Config), vp]; lib.qsl_create.restype = C.c_int
    lib.qsl_destroy.argtypes = [vp]; lib.qsl_destroy.restype = C.c_int
    lib.qsl_set_stream.argtypes = [vp, vp]; lib.qsl_set_stream.restype = C.c_int
    lib.qsl_msg_capacity_bytes.argtypes = [vp]; lib.qsl_msg_capacity_bytes.restype = C.c_size_t
    lib.qsl_compress.argtypes = [vp, vp, vp, vp, u32, u32, u64, vp, vp, vp, vp]; lib.qsl_compress.restype = C.c_int
    lib.qsl_compress_diff.argtypes = [vp, vp, vp, vp, vp, u32, u32, u64, vp, vp, vp, vp]; lib.qsl_compress_diff.restype = C.c_int
    lib.qsl_error_update.argtypes = [vp, vp, vp, vp, u32]; lib.qsl_error_update.restype = C.c_int
    lib.qsl_aggregate.argtypes = [vp, vp, C.POINTER(u32), u32, C.c_float, C.c_int, vp]; lib.qsl_aggregate.restype = C.c_int
    lib.qsl_aggregate_static.argtypes = [C.POINTER(_Config), vp, vp, C.POINTER(u32), u32, C.c_float, C.c_int, vp]
    lib.qsl_aggregate_static.restype = C.c_int
    lib.qsl_bits_sent.argtypes = [vp, vp, u32, C.POINTER(u64)]; lib.qsl_bits_sent.restype = C.c_int
    lib.qsl_device_status.argtypes = [vp]; lib.qsl_device_status.restype = C.c_int
    lib.qsl_debug_units.argtypes = [vp, C.POINTER(u32), u32, C.POINTER(u32)]; lib.qsl_debug_units.restype = C.c_int
    lib.qsl_timing_enable.argtypes = [vp, C.c_int]; lib.qsl_timing_enable.restype = C.c_int
    lib.qsl_timing_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(u32)]; lib.qsl_timing_read.restype = C.c_int
    lib.qsl_bits_index_free.argtypes = [C.POINTER(_Config), C.POINTER(u64)]; lib.qsl_bits_index_free.restype = C.c_int
    lib.qsl_plan_paths.argtypes = [C.POINTER(_Config), C.POINTER(u32)]; lib.qsl_plan_paths.restype = C.c_int
    return lib


_lib = _load()

EXPORTED = ["qsl_create", "qsl_destroy", "qsl_set_stream", "qsl_msg_capacity_bytes", "qsl_compress",
            "qsl_compress_diff", "qsl_error_update", "qsl_aggregate", "qsl_aggregate_static", "qsl_bits_sent", "qsl_bits_index_free", "qsl_plan_paths",
            "qsl_device_status", "qsl_debug_units",
            "qsl_timing_enable", "qsl_timing_read", "qsl_status_string"]


def _check(status, where):
    if status != OK:
        raise QslError(status, where)


def _ptr(t, dtype=None, allow_none=False):
    if t is None:
        if allow_none:
            return None
        raise ValueError("tensor required")
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def bits_index_free(d, seg_offset, seg_k, s, sparsifier, quantizer):
    """`qsl_bits_index_free`: bits of one Rand_k message without its indices (host only, no GPU needed)."""
    off = np.ascontiguousarray(seg_offset, dtype=np.uint64)
    k = np.ascontiguousarray(seg_k, dtype=np.uint32)
    cfg = _Config(int(d), int(k.size), off.ctypes.data_as(C.POINTER(C.c_uint64)), k.ctypes.data_as(C.POINTER(C.c_uint32)),
                  int(s), int(sparsifier), int(quantizer), 0, 1, 0)
    bits = C.c_uint64(0)
    _check(_lib.qsl_bits_index_free(C.byref(cfg), C.byref(bits)), "qsl_bits_index_free")
    return int(bits.value)


def plan_paths(d, seg_offset, seg_k, s, sparsifier, quantizer, flags=0):
    """`qsl_plan_paths`: the selection path of every segment (host only, no GPU needed)."""
    off = np.ascontiguousarray(seg_offset, dtype=np.uint64)
    k = np.ascontiguousarray(seg_k, dtype=np.uint32)
    cfg = _Config(int(d), int(k.size), off.ctypes.data_as(C.POINTER(C.c_uint64)), k.ctypes.data_as(C.POINTER(C.c_uint32)),
                  int(s), int(sparsifier), int(quantizer), 0, 1, int(flags))
    out = np.zeros(k.size, dtype=np.uint32)
    _check(_lib.qsl_plan_paths(C.byref(cfg), out.ctypes.data_as(C.POINTER(C.c_uint32))), "qsl_plan_paths")
    return out


def aggregate_static(d, k, s, sparsifier, quantizer, msg, out, scale, worker_list=None, accumulate=False):
    """`qsl_aggregate_static`: the master line without a context and without any allocation (one segment)."""
    off = np.array([0, int(d)], dtype=np.uint64)
    kk = np.array([int(k)], dtype=np.uint32)
    cfg = _Config(int(d), 1, off.ctypes.data_as(C.POINTER(C.c_uint64)), kk.ctypes.data_as(C.POINTER(C.c_uint32)),
                  int(s), int(sparsifier), int(quantizer), 0, 1, 0)
    if worker_list is None:
        R, lst = msg.shape[0], None
    else:
        lst = (C.c_uint32 * len(worker_list))(*[int(x) for x in worker_list])
        R = len(worker_list)
    stream = C.c_void_p(torch.cuda.current_stream(msg.device).cuda_stream)
    _check(_lib.qsl_aggregate_static(C.byref(cfg), stream, _ptr(msg, torch.uint8), lst, R, float(scale),
                                     int(bool(accumulate)), _ptr(out, torch.float32)), "qsl_aggregate_static")


class Qsl:
    """One operator Q Comp_k (a `qsl_ctx`).  Methods mirror the C entry points one to one."""

    def __init__(self, d, seg_offset, seg_k, s, sparsifier, quantizer, seed, max_workers, flags=0, device=None):
        self.device = torch.device("cuda" if device is None else device)
        self._off = np.ascontiguousarray(seg_offset, dtype=np.uint64)
        self._k = np.ascontiguousarray(seg_k, dtype=np.uint32)
        self.d, self.L, self.K = int(d), int(self._k.size), int(self._k.sum())
        self.s, self.sparsifier, self.quantizer, self.seed = int(s), int(sparsifier), int(quantizer), int(seed)
        self.max_workers = int(max_workers)
        cfg = _Config(self.d, self.L, self._off.ctypes.data_as(C.POINTER(C.c_uint64)),
                      self._k.ctypes.data_as(C.POINTER(C.c_uint32)), self.s, self.sparsifier, self.quantizer,
                      self.seed, self.max_workers, int(flags))
        self._ctx = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(_lib.qsl_create(C.byref(self._ctx), C.byref(cfg), self._stream()), "qsl_create")
        self.capacity = int(_lib.qsl_msg_capacity_bytes(self._ctx))

    def _stream(self):
        return C.c_void_p(torch.cuda.current_stream(self.device).cuda_stream)

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            _lib.qsl_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- allocation helpers (plumbing, not part of the C ABI) ---------------------------------
    def new_msg(self, R):
        return torch.empty(R, self.capacity, dtype=torch.uint8, device=self.device)

    # -- the C entry points -------------------------------------------------------------------
    def compress(self, m, delta, m_out, worker0, rnd, msg, msg_bits=None, sel_idx=None, sel_level=None):
        R = m.shape[0]
        assert m.shape == (R, self.d) and delta.shape == m.shape and (m_out is None or m_out.shape == m.shape)
        assert msg.shape == (R, self.capacity)
        _check(_lib.qsl_set_stream(self._ctx, self._stream()), "qsl_set_stream")
        _check(_lib.qsl_compress(self._ctx, _ptr(m, torch.float32), _ptr(delta, torch.float32),
                                 _ptr(m_out, torch.float32, True), int(worker0), R, int(rnd), _ptr(msg, torch.uint8),
                                 _ptr(msg_bits, torch.int64, True), _ptr(sel_idx, torch.int32, True),
                                 _ptr(sel_level, torch.int16, True)), "qsl_compress")

    def compress_diff(self, m, x, xhat_half, m_out, worker0, rnd, msg, msg_bits=None, sel_idx=None, sel_level=None):
        R = m.shape[0]
        assert m.shape == (R, self.d) and xhat_half.shape == m.shape and x.shape == (self.d,)
        assert m_out is None or m_out.shape == m.shape
        assert msg.shape == (R, self.capacity)
        _check(_lib.qsl_set_stream(self._ctx, self._stream()), "qsl_set_stream")
        _check(_lib.qsl_compress_diff(self._ctx, _ptr(m, torch.float32), _ptr(x, torch.float32),
                                      _ptr(xhat_half, torch.float32), _ptr(m_out, torch.float32, True), int(worker0), R,
                                      int(rnd), _ptr(msg, torch.uint8), _ptr(msg_bits, torch.int64, True),
                                      _ptr(sel_idx, torch.int32, True), _ptr(sel_level, torch.int16, True)),
               "qsl_compress_diff")

    def error_update(self, m, delta, msg):
        R = m.shape[0]
        assert m.shape == (R, self.d) and delta.shape == m.shape and msg.shape == (R, self.capacity)
        _check(_lib.qsl_set_stream(self._ctx, self._stream()), "qsl_set_stream")
        _check(_lib.qsl_error_update(self._ctx, _ptr(m, torch.float32), _ptr(delta, torch.float32),
                                     _ptr(msg, torch.uint8), R), "qsl_error_update")

    def aggregate(self, msg, out, scale, worker_list=None, accumulate=False):
        assert msg.shape[1] == self.capacity and out.shape == (self.d,)
        if worker_list is None:
            R, lst = msg.shape[0], None
        else:
            arr = (C.c_uint32 * len(worker_list))(*[int(x) for x in worker_list])
            R, lst = len(worker_list), arr
            assert max(worker_list) < msg.shape[0]
        _check(_lib.qsl_set_stream(self._ctx, self._stream()), "qsl_set_stream")
        _check(_lib.qsl_aggregate(self._ctx, _ptr(msg, torch.uint8), lst, R, float(scale), int(bool(accumulate)),
                                  _ptr(out, torch.float32)), "qsl_aggregate")

    def bits_sent(self, msg):
        R = msg.shape[0]
        out = (C.c_uint64 * R)()
        _check(_lib.qsl_set_stream(self._ctx, self._stream()), "qsl_set_stream")
        _check(_lib.qsl_bits_sent(self._ctx, _ptr(msg, torch.uint8), R, out), "qsl_bits_sent")
        return [int(x) for x in out]

    def device_status(self):
        return int(_lib.qsl_device_status(self._ctx))

    def debug_units(self):
        n = C.c_uint32()
        cap = self.max_workers * self.L
        buf = (C.c_uint32 * (8 * cap))()
        _check(_lib.qsl_debug_units(self._ctx, buf, cap, C.byref(n)), "qsl_debug_units")
        a = np.ctypeslib.as_array(buf).reshape(cap, 8)[: n.value].copy()
        return a

    def timing_enable(self, on=True):
        _check(_lib.qsl_timing_enable(self._ctx, int(on)), "qsl_timing_enable")

    def timing_read(self):
        ms, n = C.c_double(), C.c_uint32()
        _check(_lib.qsl_timing_read(self._ctx, C.byref(ms), C.byref(n)), "qsl_timing_read")
        return ms.value, n.value


def from_workload(wl, max_workers=None, flags=0, device=None) -> Qsl:
    if getattr(wl, "dense", False):
        flags |= FLAG_DENSE_FORMAT
    return Qsl(wl.d, wl.seg_offset, wl.seg_k, wl.s, wl.sparsifier, wl.quantizer, wl.seed,
               max_workers or wl.R, flags=flags, device=device)
