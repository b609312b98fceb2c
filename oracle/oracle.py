"""ctypes access to the CPU oracle (oracle/persia_oracle.cpp) -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
It never imports the HIP package; inputs arrive as numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "persia_oracle.cpp")
_LIB = os.path.join(_HERE, "libpersia_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (no fused multiply-add contraction, so the table
    initialiser's multiply and add stay two roundings)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def load(path: str):
    """Loads an oracle library from `path` and declares its prototypes (tests use this for deliberately
    broken copies of the oracle, to show that the pins notice)."""
    L = C.CDLL(path)
    _configure(L)
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = load(build())
    return _lib


def _configure(L):
    L.orc_mix64.restype = C.c_uint64
    L.orc_mix64.argtypes = [C.c_uint64]
    L.orc_round_bf16.restype = C.c_float
    L.orc_round_bf16.argtypes = [C.c_float]
    L.orc_round_bf16_once.restype = C.c_float
    L.orc_round_bf16_once.argtypes = [C.c_double]
    L.orc_init_value.restype = C.c_float
    L.orc_init_value.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32, C.c_float, C.c_float]
    L.orc_create.restype = C.c_void_p
    L.orc_create.argtypes = [C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p,
                             C.c_int, C.c_int, C.c_float, C.c_float, C.c_float, C.c_uint64, C.c_float, C.c_float,
                             C.c_int]
    L.orc_destroy.argtypes = [C.c_void_p]
    L.orc_pooled_width.restype = C.c_uint32
    L.orc_pooled_width.argtypes = [C.c_void_p]
    L.orc_rows_stored.restype = C.c_uint64
    L.orc_rows_stored.argtypes = [C.c_void_p, C.c_uint32]
    for name in ("orc_hash_rows", "orc_lookup_pool"):
        getattr(L, name).argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p]
    L.orc_dedup.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32]
    L.orc_dedup_sizes.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    L.orc_dedup_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.orc_gradient.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p]
    L.orc_grad_size.restype = C.c_uint64
    L.orc_grad_size.argtypes = [C.c_void_p]
    L.orc_grad_copy.argtypes = [C.c_void_p, C.c_void_p]
    L.orc_apply_update.argtypes = [C.c_void_p]
    L.orc_backward_update.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p]
    L.orc_read_rows.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
    L.orc_write_rows.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]


def mix64(x: int) -> int:
    return int(lib().orc_mix64(C.c_uint64(x & (2 ** 64 - 1))))


def round_bf16(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    f = lib().orc_round_bf16
    return np.array([f(C.c_float(v)) for v in x.ravel()], dtype=np.float32).reshape(x.shape)


def round_bf16_once(v: float) -> float:
    """fp64 -> bf16 in one rounding (what a bf16 table stores of an fp64 result), widened to fp32."""
    return float(lib().orc_round_bf16_once(C.c_double(v)))


def init_value(seed, t, r, dim, d, lo, hi) -> float:
    return float(lib().orc_init_value(seed, t, r, dim, d, lo, hi))


class Oracle:
    """One oracle instance = one set of tables with optimizer state.

    `tables`: list of (rows, dim, dtype) ; `slots`: list of (table, salt).
    dense=True materialises whole tables; dense=False keeps only touched rows and
    regenerates any other row from the counter-based initialiser on demand.
    """

    def __init__(self, tables, slots, hash_kind, opt, lr, eps, acc_init, init_seed, init_lo, init_hi, dense=True):
        self.L = lib()
        self.tables = [tuple(t) for t in tables]
        self.slots = [tuple(s) for s in slots]
        rows = np.array([t[0] for t in tables], dtype=np.uint64)
        dims = np.array([t[1] for t in tables], dtype=np.uint32)
        dts = np.array([t[2] for t in tables], dtype=np.int32)
        st = np.array([s[0] for s in slots], dtype=np.uint32)
        ss = np.array([s[1] for s in slots], dtype=np.uint64)
        self.h = self.L.orc_create(len(tables), rows.ctypes.data, dims.ctypes.data, dts.ctypes.data, len(slots),
                                   st.ctypes.data, ss.ctypes.data, int(hash_kind), int(opt), lr, eps, acc_init,
                                   int(init_seed), init_lo, init_hi, 1 if dense else 0)
        if not self.h:
            raise ValueError("oracle: bad configuration")
        self.S = len(slots)
        self.width = int(self.L.orc_pooled_width(self.h))

    @classmethod
    def from_config(cls, cfg, dense=True):
        """cfg: an object with the fields of workload.EmbConfig (duck-typed; not imported here)."""
        return cls([(t.rows, t.dim, t.dtype) for t in cfg.tables], [(s.table, s.salt) for s in cfg.slots],
                   cfg.hash_kind, cfg.opt, cfg.lr, cfg.eps, cfg.acc_init, cfg.init_seed, cfg.init_lo, cfg.init_hi,
                   dense=dense)

    def close(self):
        if self.h:
            self.L.orc_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _batch(ids, offsets):
        ids = np.ascontiguousarray(ids, dtype=np.uint64)
        offsets = np.ascontiguousarray(offsets, dtype=np.int32)
        return ids, offsets

    def _B(self, offsets):
        nb = len(offsets) - 1
        assert nb % self.S == 0
        return nb // self.S

    def hash_rows(self, ids, offsets):
        ids, offsets = self._batch(ids, offsets)
        out = np.empty(len(ids), dtype=np.uint32)
        self.L.orc_hash_rows(self.h, ids.ctypes.data, offsets.ctypes.data, self._B(offsets), out.ctypes.data)
        return out

    def lookup_pool(self, ids, offsets):
        ids, offsets = self._batch(ids, offsets)
        B = self._B(offsets)
        out = np.empty((B, self.width), dtype=np.float32)
        self.L.orc_lookup_pool(self.h, ids.ctypes.data, offsets.ctypes.data, B, out.ctypes.data)
        return out

    def _dedup_out(self):
        U, N = C.c_uint64(), C.c_uint64()
        self.L.orc_dedup_sizes(self.h, C.byref(U), C.byref(N))
        keys = np.empty(U.value, dtype=np.uint64)
        seg_off = np.empty(U.value + 1, dtype=np.uint32)
        seg_bags = np.empty(N.value, dtype=np.uint32)
        self.L.orc_dedup_copy(self.h, keys.ctypes.data, seg_off.ctypes.data, seg_bags.ctypes.data)
        return keys, seg_off, seg_bags

    def dedup(self, ids, offsets):
        ids, offsets = self._batch(ids, offsets)
        self.L.orc_dedup(self.h, ids.ctypes.data, offsets.ctypes.data, self._B(offsets))
        return self._dedup_out()

    def gradient(self, ids, offsets, d_pooled):
        """Ragged fp64 gradient per unique key of the batch (dedup is run first)."""
        ids, offsets = self._batch(ids, offsets)
        d_pooled = np.ascontiguousarray(d_pooled, dtype=np.float32)
        B = self._B(offsets)
        assert d_pooled.shape == (B, self.width)
        self.L.orc_dedup(self.h, ids.ctypes.data, offsets.ctypes.data, B)
        self.L.orc_gradient(self.h, B, d_pooled.ctypes.data)
        return self.last_gradient()

    def last_gradient(self):
        g = np.empty(int(self.L.orc_grad_size(self.h)), dtype=np.float64)
        self.L.orc_grad_copy(self.h, g.ctypes.data)
        return g

    def backward_update(self, ids, offsets, d_pooled):
        ids, offsets = self._batch(ids, offsets)
        d_pooled = np.ascontiguousarray(d_pooled, dtype=np.float32)
        B = self._B(offsets)
        assert d_pooled.shape == (B, self.width)
        self.L.orc_backward_update(self.h, ids.ctypes.data, offsets.ctypes.data, B, d_pooled.ctypes.data)
        return self._dedup_out()

    def read_rows(self, table, rows):
        rows = np.ascontiguousarray(rows, dtype=np.uint64)
        D = self.tables[table][1]
        w = np.empty((len(rows), D), dtype=np.float32)
        a = np.empty(len(rows), dtype=np.float32)
        rc = self.L.orc_read_rows(self.h, table, rows.ctypes.data, len(rows), w.ctypes.data, a.ctypes.data)
        if rc:
            raise ValueError("read_rows: bad table or row")
        return w, a

    def write_rows(self, table, rows, w, acc=None):
        rows = np.ascontiguousarray(rows, dtype=np.uint64)
        w = np.ascontiguousarray(w, dtype=np.float32)
        assert w.shape == (len(rows), self.tables[table][1])
        ap = None
        if acc is not None:
            acc = np.ascontiguousarray(acc, dtype=np.float32)
            ap = acc.ctypes.data
        rc = self.L.orc_write_rows(self.h, table, rows.ctypes.data, len(rows), w.ctypes.data, ap)
        if rc:
            raise ValueError("write_rows: bad table or row")

    def rows_stored(self, table):
        return int(self.L.orc_rows_stored(self.h, table))
