"""ctypes loader for the CPU oracle (test infrastructure, not product code).

Only tests, ``__graft_entry__.smoke()`` and the CPU-baseline leg of ``bench.py``
may import this module.  It builds ``libctr_oracle.so`` next to the source with
g++ when the library is missing or older than the source.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ctr_oracle.cpp")
_LIB = os.path.join(_HERE, "libctr_oracle.so")

OK, E_INVAL, E_NOMEM, E_FULL, E_BADKEY, E_STATE = 0, 1, 2, 3, 4, 5
STEP_LOCAL, STEP_MERGE_PENDING = 0, 1
VAR_ALG2, VAR_ADAGRAD, VAR_PROSE, VAR_KINGMA = 0, 1, 2, 3


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-Wall",
               "-o", _LIB, _SRC]
        subprocess.check_call(cmd)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        u64, u32, f32, vp = C.c_uint64, C.c_uint32, C.c_float, C.c_void_p
        L.orc_create.restype = vp
        L.orc_create.argtypes = [u64, u32, u32, f32, f32, f32, f32, u64, f32, C.c_int, C.c_int]
        L.orc_destroy.argtypes = [vp]
        L.orc_n_rows.restype = u64
        L.orc_n_rows.argtypes = [vp]
        L.orc_batch_n_unique.restype = u64
        L.orc_batch_n_unique.argtypes = [vp]
        L.orc_batch_n_new.restype = u64
        L.orc_batch_n_new.argtypes = [vp]
        L.orc_init_value.restype = f32
        L.orc_init_value.argtypes = [u64, u64, u32, f32]
        L.orc_lookup.restype = C.c_int64
        L.orc_lookup.argtypes = [vp, u64]
        L.orc_pull_pool.restype = C.c_int
        L.orc_pull_pool.argtypes = [vp, u32, vp, u64, vp, u32, vp]
        L.orc_push_adam.restype = C.c_int
        L.orc_push_adam.argtypes = [vp, u32, vp, u32]
        L.orc_kstep_merge.restype = C.c_int
        L.orc_kstep_merge.argtypes = [vp]
        L.orc_batch_export.restype = C.c_int
        L.orc_batch_export.argtypes = [vp, vp, vp, vp]
        L.orc_table_export.restype = C.c_int
        L.orc_table_export.argtypes = [vp, u32, vp, vp, vp, vp, vp]
        L.orc_table_load.restype = C.c_int
        L.orc_table_load.argtypes = [vp, vp, u64, vp, vp, vp]
        L.orc_lookup_pool.restype = C.c_int
        L.orc_lookup_pool.argtypes = [vp, u32, vp, u64, vp, u32, vp]
        L.orc_table_clear.restype = C.c_int
        L.orc_table_clear.argtypes = [vp]
        L.orc_table_collect.restype = C.c_int
        L.orc_table_collect.argtypes = [vp, u32, vp, u64, vp, vp, vp, vp]
        _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def init_value(seed: int, key: int, d: int, init_std: float) -> float:
    return float(lib().orc_init_value(seed, key, d, init_std))


class OracleTable:
    """One table (W replicas sharing a key->row map) held in host memory."""

    def __init__(self, capacity_rows, dim, n_replicas=1, lr=1e-3, beta1=0.9, beta2=0.999,
                 eps=1e-8, init_seed=0, init_std=0.01, kstep=False, variant=VAR_ALG2):
        self.R, self.D, self.W, self.kstep = int(capacity_rows), int(dim), int(n_replicas), bool(kstep)
        self.variant = int(variant)
        self._h = lib().orc_create(self.R, self.D, self.W, lr, beta1, beta2, eps, init_seed,
                                   init_std, int(self.kstep), self.variant)
        if not self._h:
            raise ValueError("bad oracle table parameters")

    def close(self):
        if self._h:
            lib().orc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def n_rows(self) -> int:
        return int(lib().orc_n_rows(self._h))

    @property
    def n_new_last(self) -> int:
        return int(lib().orc_batch_n_new(self._h))

    def lookup(self, key: int) -> int:
        return int(lib().orc_lookup(self._h, int(key)))

    def pull_pool(self, replica, keys, offsets):
        """Returns (status, pooled[G, D] float32)."""
        keys = np.ascontiguousarray(keys, dtype=np.uint64)
        offsets = np.ascontiguousarray(offsets, dtype=np.uint32)
        G = offsets.size - 1
        pooled = np.zeros((G, self.D), dtype=np.float32)
        st = lib().orc_pull_pool(self._h, replica, _ptr(keys), keys.size, _ptr(offsets), G,
                                 _ptr(pooled))
        return st, pooled

    def push_adam(self, replica, grad, mode=STEP_LOCAL):
        grad = np.ascontiguousarray(grad, dtype=np.float32)
        return lib().orc_push_adam(self._h, replica, _ptr(grad), mode)

    def kstep_merge(self):
        return lib().orc_kstep_merge(self._h)

    def table_load(self, keys, x, m, v):
        keys = np.ascontiguousarray(keys, dtype=np.uint64)
        x = np.ascontiguousarray(x, dtype=np.float32)
        v = np.ascontiguousarray(v, dtype=np.float32)
        m = np.zeros_like(x) if m is None else np.ascontiguousarray(m, dtype=np.float32)
        return lib().orc_table_load(self._h, _ptr(keys), keys.size, _ptr(x), _ptr(m), _ptr(v))

    def lookup_pool(self, replica, keys, offsets):
        """(status, pooled[G, D]) without inserting: absent keys contribute nothing."""
        keys = np.ascontiguousarray(keys, dtype=np.uint64)
        offsets = np.ascontiguousarray(offsets, dtype=np.uint32)
        n_seg = offsets.size - 1
        pooled = np.zeros((n_seg, self.D), np.float32)
        st = lib().orc_lookup_pool(self._h, replica, _ptr(keys), keys.size, _ptr(offsets), n_seg, _ptr(pooled))
        return st, pooled

    def table_clear(self):
        return lib().orc_table_clear(self._h)

    def table_collect(self, replica, keys):
        """(status, x, m, v, found) for the given keys, without inserting."""
        keys = np.ascontiguousarray(keys, dtype=np.uint64)
        n = keys.size
        x = np.empty((n, self.D), np.float32)
        m = np.empty((n, self.D), np.float32)
        v = np.empty((n, self.D), np.float32)
        found = np.empty(n, np.uint32)
        st = lib().orc_table_collect(self._h, replica, _ptr(keys), n, _ptr(x), _ptr(m), _ptr(v), _ptr(found))
        return st, x, m, v, found

    def batch_export(self, n_keys):
        """(uniq ascending, rows, inverse) of the last pull; call before the push."""
        U = int(lib().orc_batch_n_unique(self._h))
        uniq = np.empty(U, np.uint64)
        rows = np.empty(U, np.uint32)
        inv = np.empty(int(n_keys), np.uint32)
        st = lib().orc_batch_export(self._h, _ptr(uniq), _ptr(rows), _ptr(inv))
        if st != OK:
            raise RuntimeError("no live batch")
        return uniq, rows, inv

    def table_export(self, replica=0):
        """dict(keys[n], x[n,D], m[n,D], v[n,D], vhat[n,D] or None) in row order."""
        n = self.n_rows
        keys = np.empty(n, np.uint64)
        x = np.empty((n, self.D), np.float32)
        m = np.empty((n, self.D), np.float32)
        v = np.empty((n, self.D), np.float32)
        vhat = np.empty((n, self.D), np.float32) if (self.kstep and self.variant != VAR_PROSE) else None
        st = lib().orc_table_export(self._h, replica, _ptr(keys), _ptr(x), _ptr(m), _ptr(v),
                                    _ptr(vhat) if vhat is not None else None)
        if st != OK:
            raise RuntimeError("table_export failed: %d" % st)
        return {"keys": keys, "x": x, "m": m, "v": v, "vhat": vhat}
