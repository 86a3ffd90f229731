"""ctypes front-end of the CPU oracle (`qsl_oracle.cpp`).

TEST INFRASTRUCTURE ONLY: imported by `tests/`, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU package never imports this module and
this module never imports the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qsl_oracle.cpp")
_LIB = os.path.join(_HERE, "libqsl_oracle.so")

TOPK, RANDK = 0, 1
QSGD, SIGN_L1, SIGN_L2, FP32, QSGD_SCALED, SIGN_L3, SIGN_L4 = 0, 1, 2, 3, 4, 5, 6
DENSE_FORMAT = 0x100          # added to the quantiser number: the index-free format of an operator that keeps every coordinate
STREAM_SELECT, STREAM_QUANT = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler; returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        u8p, u16p, u32p, u64p, f32p = (C.POINTER(t) for t in (C.c_uint8, C.c_uint16, C.c_uint32, C.c_uint64, C.c_float))
        L.qslo_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.qslo_philox4x32_10.restype = None
        L.qslo_random_word.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint64]
        L.qslo_random_word.restype = C.c_uint32
        L.qslo_exact_sum_of_squares.argtypes = [f32p, C.c_uint64]
        L.qslo_exact_sum_of_squares.restype = C.c_double
        L.qslo_exact_sum_of_abs.argtypes = [f32p, C.c_uint64]
        L.qslo_exact_sum_of_abs.restype = C.c_double
        lay = [C.c_uint64, C.c_uint32, u64p, u32p, C.c_uint32, C.c_uint32]
        L.qslo_msg_capacity_bytes.argtypes = lay
        L.qslo_msg_capacity_bytes.restype = C.c_uint64
        L.qslo_compress.argtypes = [f32p, f32p, f32p, C.c_uint64, C.c_uint32, u64p, u32p, C.c_uint32, C.c_uint32,
                                    C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint64, u8p, C.c_uint64, u64p, u32p,
                                    u16p, u8p, f32p, f32p]
        L.qslo_compress.restype = C.c_int
        L.qslo_bits_sent.argtypes = [u8p] + lay
        L.qslo_bits_sent.restype = C.c_uint64
        L.qslo_decode.argtypes = [u8p] + lay + [u32p, f32p, C.c_uint64]
        L.qslo_decode.restype = C.c_int64
        L.qslo_error_update.argtypes = [f32p, f32p, u8p] + lay
        L.qslo_error_update.restype = C.c_int
        L.qslo_aggregate.argtypes = [u8p, C.c_uint64, u32p, C.c_uint32, C.c_float, C.c_int, f32p] + lay
        L.qslo_aggregate.restype = C.c_int
        _lib = L
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    o = np.zeros(4, dtype=np.uint32)
    lib().qslo_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(o, C.c_uint32))
    return o


def random_word(seed, worker, rnd, stream, i):
    return int(lib().qslo_random_word(seed, worker, rnd, stream, i))


def exact_sum_of_squares(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    return float(lib().qslo_exact_sum_of_squares(_p(x, C.c_float), x.size))


def exact_sum_of_abs(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    return float(lib().qslo_exact_sum_of_abs(_p(x, C.c_float), x.size))


class OracleOp:
    """The operator Q Comp_k with its parameters fixed; one worker per call."""

    def __init__(self, d, seg_offset, seg_k, s, sparsifier, quantizer, seed, dense=False):
        self.d = int(d)
        self.off = np.ascontiguousarray(seg_offset, dtype=np.uint64)
        self.k = np.ascontiguousarray(seg_k, dtype=np.uint32)
        self.L = int(self.k.size)
        self.s = int(s)
        self.sparsifier = int(sparsifier)
        self.quantizer = int(quantizer)
        self.dense = bool(dense)
        self._qarg = self.quantizer | (DENSE_FORMAT if self.dense else 0)
        self.seed = int(seed)
        self.K = int(self.k.sum())
        self._lay = (self.d, self.L, _p(self.off, C.c_uint64), _p(self.k, C.c_uint32), self.s, self._qarg)
        self.capacity = int(lib().qslo_msg_capacity_bytes(*self._lay))
        if self.capacity == 0:
            raise ValueError("invalid operator parameters")

    def compress(self, m, delta, worker, rnd, want_m_out=True):
        m = np.ascontiguousarray(m, dtype=np.float32)
        delta = np.ascontiguousarray(delta, dtype=np.float32)
        assert m.size == self.d and delta.size == self.d
        m_out = np.empty(self.d, dtype=np.float32) if want_m_out else None
        msg = np.zeros(self.capacity, dtype=np.uint8)
        bits = np.zeros(1, dtype=np.uint64)
        sel_idx = np.zeros(self.K, dtype=np.uint32)
        sel_level = np.zeros(self.K, dtype=np.uint16)
        sel_neg = np.zeros(self.K, dtype=np.uint8)
        scales = np.zeros(self.L, dtype=np.float32)
        g_val = np.zeros(self.K, dtype=np.float32)
        rc = lib().qslo_compress(_p(m, C.c_float), _p(delta, C.c_float), _p(m_out, C.c_float), self.d, self.L,
                                 _p(self.off, C.c_uint64), _p(self.k, C.c_uint32), self.s, self.sparsifier,
                                 self._qarg, self.seed, int(worker), int(rnd), _p(msg, C.c_uint8), self.capacity,
                                 _p(bits, C.c_uint64), _p(sel_idx, C.c_uint32), _p(sel_level, C.c_uint16),
                                 _p(sel_neg, C.c_uint8), _p(scales, C.c_float), _p(g_val, C.c_float))
        if rc != 0:
            raise RuntimeError(f"qslo_compress failed with status {rc}")
        return dict(m_out=m_out, msg=msg, bits=int(bits[0]), sel_idx=sel_idx, sel_level=sel_level, sel_neg=sel_neg,
                    scales=scales, g_val=g_val)

    def compress_diff(self, m, x, xhat_half, worker, rnd):
        """The synchronisation line of Algorithm 1 as written: g = Q Comp_k(m + x_t - xhat_{t+1/2}), the
        difference taken first, in fp32."""
        x = np.ascontiguousarray(x, dtype=np.float32)
        xhat_half = np.ascontiguousarray(xhat_half, dtype=np.float32)
        return self.compress(m, np.subtract(x, xhat_half, dtype=np.float32), worker, rnd)

    def bits_index_free(self):
        """Accounting variant for Rand_k (Section 2.2: the k-subset does not depend on the data, so common
        randomness lets the receiver rebuild it): a message without indices holds one fp32 scale per segment
        and, for each of the K chosen coordinates, one code -- written out as a sum over the coordinates."""
        if self.sparsifier != RANDK:
            raise ValueError("only Rand_k can drop its indices")
        bits = 0
        for _segment in range(self.L):
            bits += 32                                   # the scale
        for _coordinate in range(self.K):
            if self.quantizer == FP32:
                bits += 32
            elif self.quantizer in (SIGN_L1, SIGN_L2, SIGN_L3, SIGN_L4):
                bits += 1
            else:
                bits += len(format(self.s, "b")) + 1     # a level in 0..s, then the sign
        return bits

    def bits_sent(self, msg):
        msg = np.ascontiguousarray(msg, dtype=np.uint8)
        return int(lib().qslo_bits_sent(_p(msg, C.c_uint8), *self._lay))

    def decode(self, msg):
        msg = np.ascontiguousarray(msg, dtype=np.uint8)
        idx = np.zeros(self.K, dtype=np.uint32)
        val = np.zeros(self.K, dtype=np.float32)
        n = lib().qslo_decode(_p(msg, C.c_uint8), *self._lay, _p(idx, C.c_uint32), _p(val, C.c_float), self.K)
        if n < 0:
            raise RuntimeError("qslo_decode: inconsistent message")
        return idx[:n].copy(), val[:n].copy()

    def error_update(self, m, delta, msg):
        m = np.array(m, dtype=np.float32, copy=True)
        delta = np.ascontiguousarray(delta, dtype=np.float32)
        msg = np.ascontiguousarray(msg, dtype=np.uint8)
        rc = lib().qslo_error_update(_p(m, C.c_float), _p(delta, C.c_float), _p(msg, C.c_uint8), *self._lay)
        if rc != 0:
            raise RuntimeError(f"qslo_error_update failed with status {rc}")
        return m

    def aggregate(self, msgs, scale, worker_list=None, out=None):
        """msgs: [R_total, capacity] uint8.  Returns the dense d-vector."""
        msgs = np.ascontiguousarray(msgs, dtype=np.uint8)
        assert msgs.ndim == 2 and msgs.shape[1] == self.capacity
        lst = None if worker_list is None else np.ascontiguousarray(worker_list, dtype=np.uint32)
        R = msgs.shape[0] if lst is None else lst.size
        accumulate = out is not None
        res = np.array(out, dtype=np.float32, copy=True) if accumulate else np.zeros(self.d, dtype=np.float32)
        rc = lib().qslo_aggregate(_p(msgs, C.c_uint8), self.capacity, _p(lst, C.c_uint32), R, float(scale),
                                  int(accumulate), _p(res, C.c_float), *self._lay)
        if rc != 0:
            raise RuntimeError(f"qslo_aggregate failed with status {rc}")
        return res
