"""Thin ctypes binding of the C ABI in include/ctr_sparse.h (argument marshalling only).

The functions carry the ABI's names and take raw device addresses; ``CtrTable``
is a convenience that owns the torch allocations (device memory and the stream
come from PyTorch, nothing else does).  There is no fallback: if the HIP
library is not built, importing the symbols raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# CTR_SPARSE_LIB: another build of the same library (a compile-time variant made by build.py --define ... --out),
# for A/B measurements; it must exist, like the in-tree one
LIB_PATH = os.environ.get("CTR_SPARSE_LIB") or os.path.join(_HERE, "libctr_sparse.so")

CTR_OK, CTR_E_INVAL, CTR_E_NOMEM, CTR_E_FULL, CTR_E_BADKEY, CTR_E_STATE, CTR_E_DEVICE = range(7)
CTR_F_KSTEP, CTR_F_ADAGRAD, CTR_F_KSTEP_PROSE, CTR_F_BIAS_CORRECTION = 1, 2, 4, 8
CTR_STEP_LOCAL, CTR_STEP_MERGE_PENDING = 0, 1
CTR_N_STAGES = 8
CTR_NOALLOC_MAX_KEYS = 1 << 22
STAGE_NAMES = ("probe", "insert", "pool", "sort", "push", "fixup", "merge", "order")

EXPORTED = (
    "ctr_table_bytes", "ctr_workspace_bytes", "ctr_table_create", "ctr_table_destroy",
    "ctr_pull_pool", "ctr_pull_pool_bf16", "ctr_lookup_pool", "ctr_lookup_pool_noalloc", "ctr_push_adam", "ctr_push_adam_bf16", "ctr_kstep_merge", "ctr_table_load", "ctr_table_collect", "ctr_table_clear",
    "ctr_table_size", "ctr_table_export",
    "ctr_batch_export", "ctr_batch_stats", "ctr_merge_stats", "ctr_stream_copy", "ctr_last_status", "ctr_debug_set_geometry", "ctr_debug_set_push_order", "ctr_profile_enable",
    "ctr_profile_read",
)


class ctr_config(C.Structure):
    _fields_ = [
        ("capacity_rows", C.c_uint64),
        ("dim", C.c_uint32),
        ("load_factor", C.c_float),
        ("n_replicas", C.c_uint32),
        ("lr", C.c_float),
        ("beta1", C.c_float),
        ("beta2", C.c_float),
        ("eps", C.c_float),
        ("init_seed", C.c_uint64),
        ("init_std", C.c_float),
        ("flags", C.c_uint32),
    ]


_lib = None


def lib():
    """Loads libctr_sparse.so; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "HIP library %s is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(hipcc, gfx950) first" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, u64, u32, sz, ci = C.c_void_p, C.c_uint64, C.c_uint32, C.c_size_t, C.c_int
    cfgp = C.POINTER(ctr_config)
    L.ctr_table_bytes.restype = sz
    L.ctr_table_bytes.argtypes = [cfgp]
    L.ctr_workspace_bytes.restype = sz
    L.ctr_workspace_bytes.argtypes = [cfgp, u64, u32]
    L.ctr_table_create.restype = ci
    L.ctr_table_create.argtypes = [cfgp, vp, sz, vp, C.POINTER(vp)]
    L.ctr_table_destroy.restype = ci
    L.ctr_table_destroy.argtypes = [vp]
    L.ctr_pull_pool.restype = ci
    L.ctr_pull_pool.argtypes = [vp, u32, vp, u64, vp, u32, vp, vp, sz, C.POINTER(vp), vp]
    L.ctr_debug_set_geometry.restype = ci
    L.ctr_debug_set_geometry.argtypes = [vp, u32, u32]
    L.ctr_debug_set_push_order.restype = ci
    L.ctr_debug_set_push_order.argtypes = [vp, u32, u32, u64]
    L.ctr_lookup_pool.restype = ci
    L.ctr_lookup_pool.argtypes = [vp, u32, vp, u64, vp, u32, vp, vp, vp, sz, vp]
    L.ctr_lookup_pool_noalloc.restype = ci
    L.ctr_lookup_pool_noalloc.argtypes = [vp, u32, vp, u64, vp, u32, vp, vp, vp]
    L.ctr_table_clear.restype = ci
    L.ctr_table_clear.argtypes = [vp, vp]
    L.ctr_pull_pool_bf16.restype = ci
    L.ctr_pull_pool_bf16.argtypes = [vp, u32, vp, u64, vp, u32, vp, vp, vp, sz, C.POINTER(vp), vp]
    L.ctr_push_adam.restype = ci
    L.ctr_push_adam.argtypes = [vp, u32, vp, vp, u32, vp]
    L.ctr_push_adam_bf16.restype = ci
    L.ctr_push_adam_bf16.argtypes = [vp, u32, vp, vp, u32, vp]
    L.ctr_kstep_merge.restype = ci
    L.ctr_kstep_merge.argtypes = [vp, vp]
    L.ctr_table_load.restype = ci
    L.ctr_table_load.argtypes = [vp, vp, u64, vp, vp, vp, vp, sz, vp]
    L.ctr_table_collect.restype = ci
    L.ctr_table_collect.argtypes = [vp, u32, vp, u64, vp, vp, vp, vp, vp]
    L.ctr_table_size.restype = ci
    L.ctr_table_size.argtypes = [vp, C.POINTER(u64), vp]
    L.ctr_table_export.restype = ci
    L.ctr_table_export.argtypes = [vp, u32, vp, vp, vp, vp, vp, vp]
    L.ctr_batch_export.restype = ci
    L.ctr_batch_export.argtypes = [vp, vp, C.POINTER(u64), vp, vp, vp, vp]
    L.ctr_batch_stats.restype = ci
    L.ctr_batch_stats.argtypes = [vp, C.POINTER(u64), C.POINTER(u64), vp]
    L.ctr_last_status.restype = ci
    L.ctr_last_status.argtypes = [vp, vp]
    L.ctr_merge_stats.restype = ci
    L.ctr_merge_stats.argtypes = [vp, C.POINTER(u64), C.POINTER(u64), vp]
    L.ctr_stream_copy.restype = ci
    L.ctr_stream_copy.argtypes = [vp, vp, sz, ci, vp]
    L.ctr_profile_enable.restype = ci
    L.ctr_profile_enable.argtypes = [vp, ci]
    L.ctr_profile_read.restype = ci
    L.ctr_profile_read.argtypes = [vp, vp, vp]
    _lib = L
    return L


# ---- the ABI's calls under their own names (raw addresses in, status out) ----

def ctr_table_bytes(cfg: ctr_config) -> int:
    return int(lib().ctr_table_bytes(C.byref(cfg)))


def ctr_workspace_bytes(cfg: ctr_config, max_keys: int, max_segments: int) -> int:
    return int(lib().ctr_workspace_bytes(C.byref(cfg), max_keys, max_segments))


def ctr_table_create(cfg: ctr_config, d_mem: int, nbytes: int, stream: int):
    out = C.c_void_p()
    st = lib().ctr_table_create(C.byref(cfg), d_mem, nbytes, stream, C.byref(out))
    return st, out.value


def ctr_table_destroy(table: int) -> int:
    return lib().ctr_table_destroy(table)


def ctr_pull_pool(table, replica, d_keys, n_keys, d_offsets, n_segments, d_pooled, d_ws, ws_bytes, stream):
    out = C.c_void_p()
    st = lib().ctr_pull_pool(table, replica, d_keys, n_keys, d_offsets, n_segments, d_pooled, d_ws,
                             ws_bytes, C.byref(out), stream)
    return st, out.value


def ctr_pull_pool_bf16(table, replica, d_keys, n_keys, d_offsets, n_segments, d_pooled, d_pooled_bf16, d_ws,
                       ws_bytes, stream):
    out = C.c_void_p()
    st = lib().ctr_pull_pool_bf16(table, replica, d_keys, n_keys, d_offsets, n_segments, d_pooled, d_pooled_bf16,
                                  d_ws, ws_bytes, C.byref(out), stream)
    return st, out.value


def ctr_lookup_pool_noalloc(table, replica, d_keys, n_keys, d_offsets, n_segments, d_pooled, d_pooled_bf16,
                            stream) -> int:
    return lib().ctr_lookup_pool_noalloc(table, replica, d_keys, n_keys, d_offsets, n_segments, d_pooled,
                                         d_pooled_bf16, stream)


def ctr_push_adam(table, replica, batch, d_grad, mode, stream) -> int:
    return lib().ctr_push_adam(table, replica, batch, d_grad, mode, stream)


def ctr_kstep_merge(table, stream) -> int:
    return lib().ctr_kstep_merge(table, stream)


def ctr_table_load(table, d_keys, n_keys, d_x, d_m, d_v, d_ws, ws_bytes, stream) -> int:
    return lib().ctr_table_load(table, d_keys, n_keys, d_x, d_m, d_v, d_ws, ws_bytes, stream)


def ctr_table_collect(table, replica, d_keys, n_keys, d_x, d_m, d_v, d_found, stream) -> int:
    return lib().ctr_table_collect(table, replica, d_keys, n_keys, d_x, d_m, d_v, d_found, stream)


def ctr_stream_copy(d_dst, d_src, nbytes, non_temporal, stream) -> int:
    return lib().ctr_stream_copy(d_dst, d_src, nbytes, 1 if non_temporal else 0, stream)


def ctr_last_status(table, stream) -> int:
    return lib().ctr_last_status(table, stream)


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class CtrTable:
    """Owns the torch allocations for one table and forwards to the ABI."""

    def __init__(self, capacity_rows, dim, n_replicas=1, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8,
                 init_seed=0, init_std=0.01, kstep=False, load_factor=0.5, max_keys=0, max_segments=0,
                 device="cuda:0", adagrad=False, prose=False, bias_correction=False):
        import torch
        self._torch = torch
        self.device = torch.device(device)
        self.cfg = ctr_config(capacity_rows, dim, load_factor, n_replicas, lr, beta1, beta2, eps,
                              init_seed, init_std,
                              (CTR_F_KSTEP if kstep else 0) | (CTR_F_ADAGRAD if adagrad else 0) |
                              (CTR_F_KSTEP_PROSE if prose else 0) |
                              (CTR_F_BIAS_CORRECTION if bias_correction else 0))
        self.D, self.W, self.R, self.kstep = int(dim), int(n_replicas), int(capacity_rows), bool(kstep)
        self.adagrad, self.prose = bool(adagrad), bool(prose)
        nbytes = ctr_table_bytes(self.cfg)
        if nbytes == 0:
            raise ValueError("invalid table configuration")
        self.table_bytes = nbytes
        self._mem = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self._ws = None
        self._ws_of_live_batch = None
        self.ws_bytes = 0
        self._handle = None
        st, h = ctr_table_create(self.cfg, self._mem.data_ptr(), nbytes, self.stream)
        if st != CTR_OK:
            raise RuntimeError("ctr_table_create failed: %d" % st)
        self._handle = h
        if max_keys:
            self.reserve(max_keys, max_segments)

    @property
    def stream(self) -> int:
        return int(self._torch.cuda.current_stream(self.device).cuda_stream)

    def reserve(self, max_keys: int, max_segments: int):
        need = ctr_workspace_bytes(self.cfg, max_keys, max_segments)
        if need == 0:
            raise ValueError("invalid workspace request")
        need += getattr(self, "_ws_slack", 0)
        if need > self.ws_bytes:
            self._torch.cuda.synchronize(self.device)
            # a batch that was pulled and not yet pushed keeps its lists in the old workspace: that
            # tensor stays alive until the next pull makes the batch stale
            self._ws_of_live_batch = self._ws
            self._ws = self._torch.empty(need, dtype=self._torch.uint8, device=self.device)
            self.ws_bytes = need

    def close(self):
        if self._handle:
            self._torch.cuda.synchronize(self.device)
            ctr_table_destroy(self._handle)
            self._handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- hot path
    def pull_pool(self, replica, keys, offsets, pooled=None):
        """keys: int64/uint64 device tensor [L]; offsets: int32 device tensor [G+1].
        Returns (status, batch handle, pooled[G, D])."""
        torch = self._torch
        n_keys, n_seg = keys.numel(), offsets.numel() - 1
        self.reserve(max(n_keys, 1), n_seg)
        self._ws_of_live_batch = None              # the previous batch goes stale with this pull
        if pooled is None:
            pooled = torch.empty((n_seg, self.D), dtype=torch.float32, device=self.device)
        st, batch = ctr_pull_pool(self._handle, replica, keys.data_ptr() if n_keys else None, n_keys,
                                  offsets.data_ptr(), n_seg, pooled.data_ptr() if n_seg else None,
                                  self._ws.data_ptr(), self.ws_bytes, self.stream)
        return st, batch, pooled

    def pull_pool_bf16(self, replica, keys, offsets, pooled_bf16=None, pooled=None, want_f32=False):
        """As pull_pool with the pooled embeddings as bfloat16 [G, D] (and as fp32 too if `pooled` is given or
        want_f32).  Returns (status, batch handle, pooled_bf16, pooled or None)."""
        torch = self._torch
        n_keys, n_seg = keys.numel(), offsets.numel() - 1
        self.reserve(max(n_keys, 1), n_seg)
        self._ws_of_live_batch = None
        if pooled_bf16 is None:
            pooled_bf16 = torch.empty((n_seg, self.D), dtype=torch.bfloat16, device=self.device)
        if pooled is None and want_f32:
            pooled = torch.empty((n_seg, self.D), dtype=torch.float32, device=self.device)
        st, batch = ctr_pull_pool_bf16(self._handle, replica, keys.data_ptr() if n_keys else None, n_keys,
                                       offsets.data_ptr(), n_seg,
                                       pooled.data_ptr() if (pooled is not None and n_seg) else None,
                                       pooled_bf16.data_ptr() if n_seg else None, self._ws.data_ptr(), self.ws_bytes,
                                       self.stream)
        return st, batch, pooled_bf16, pooled

    def lookup_pool(self, replica, keys, offsets, bf16=False, out=None):
        """Pooling without insert (prediction).  Returns (status, pooled[G, D] fp32 or bf16)."""
        torch = self._torch
        n_keys, n_seg = keys.numel(), offsets.numel() - 1
        self.reserve(max(n_keys, 1), n_seg)
        if out is not None:
            bf16 = out.dtype == torch.bfloat16
        pooled = out if out is not None else torch.empty(
            (n_seg, self.D), dtype=torch.bfloat16 if bf16 else torch.float32, device=self.device)
        ptr = pooled.data_ptr() if n_seg else None
        st = lib().ctr_lookup_pool(self._handle, replica, keys.data_ptr() if n_keys else None, n_keys,
                                   offsets.data_ptr(), n_seg, None if bf16 else ptr, ptr if bf16 else None,
                                   self._ws.data_ptr(), self.ws_bytes, self.stream)
        return st, pooled

    def push_adam(self, replica, batch, grad, mode=CTR_STEP_LOCAL):
        """grad: float32 or bfloat16 [n_seg, D] device tensor (the dtype picks the entry point)."""
        ptr = grad.data_ptr() if grad.numel() else None
        if grad.dtype == self._torch.bfloat16:
            return lib().ctr_push_adam_bf16(self._handle, replica, batch, ptr, mode, self.stream)
        return ctr_push_adam(self._handle, replica, batch, ptr, mode, self.stream)

    def kstep_merge(self):
        return ctr_kstep_merge(self._handle, self.stream)

    def table_load(self, keys, x, m, v):
        """keys int64/uint64 [n]; x, m, v float32 [n, D] device tensors (m may be None for AdaGrad rows)."""
        n = keys.numel()
        self.reserve(max(n, 1), 0)
        return ctr_table_load(self._handle, keys.data_ptr() if n else None, n, x.data_ptr() if n else None,
                              m.data_ptr() if (m is not None and n) else None, v.data_ptr() if n else None,
                              self._ws.data_ptr(), self.ws_bytes, self.stream)

    def table_clear(self):
        return lib().ctr_table_clear(self._handle, self.stream)

    def table_collect(self, replica, keys):
        """Returns (status, x, m or None, v, found) device tensors for the given keys (no insert)."""
        torch = self._torch
        n = keys.numel()
        x = torch.empty((n, self.D), dtype=torch.float32, device=self.device)
        m = None if self.adagrad else torch.empty_like(x)
        v = torch.empty_like(x)
        found = torch.empty(n, dtype=torch.int32, device=self.device)
        st = ctr_table_collect(self._handle, replica, keys.data_ptr() if n else None, n, x.data_ptr(),
                               m.data_ptr() if m is not None else None, v.data_ptr(), found.data_ptr(),
                               self.stream)
        return st, x, m, v, found

    # -- debug / parity surface
    def last_status(self) -> int:
        return ctr_last_status(self._handle, self.stream)

    @property
    def n_rows(self) -> int:
        n = C.c_uint64()
        st = lib().ctr_table_size(self._handle, C.byref(n), self.stream)
        if st != CTR_OK:
            raise RuntimeError("ctr_table_size: %d" % st)
        return int(n.value)

    def batch_stats(self):
        u, n = C.c_uint64(), C.c_uint64()
        st = lib().ctr_batch_stats(self._handle, C.byref(u), C.byref(n), self.stream)
        if st != CTR_OK:
            raise RuntimeError("ctr_batch_stats: %d" % st)
        return int(u.value), int(n.value)

    def merge_stats(self):
        """(rows merged, pending (row, replica) steps applied) by all merges so far."""
        n, q = C.c_uint64(), C.c_uint64()
        st = lib().ctr_merge_stats(self._handle, C.byref(n), C.byref(q), self.stream)
        if st != CTR_OK:
            raise RuntimeError("ctr_merge_stats: %d" % st)
        return int(n.value), int(q.value)

    def batch_export(self, batch, n_keys):
        nu = C.c_uint64()
        st = lib().ctr_batch_export(self._handle, batch, C.byref(nu), None, None, None, self.stream)
        if st != CTR_OK:
            raise RuntimeError("ctr_batch_export: %d" % st)
        U = int(nu.value)
        uniq = np.empty(U, np.uint64)
        rows = np.empty(U, np.uint32)
        inv = np.empty(int(n_keys), np.uint32)
        st = lib().ctr_batch_export(self._handle, batch, C.byref(nu), _np_ptr(uniq), _np_ptr(rows),
                                    _np_ptr(inv), self.stream)
        if st != CTR_OK:
            raise RuntimeError("ctr_batch_export: %d" % st)
        return uniq, rows, inv

    def table_export(self, replica=0):
        n = self.n_rows
        keys = np.empty(n, np.uint64)
        x = np.empty((n, self.D), np.float32)
        m = None if self.adagrad else np.empty((n, self.D), np.float32)
        v = np.empty((n, self.D), np.float32)
        vhat = np.empty((n, self.D), np.float32) if (self.kstep and not self.prose) else None
        st = lib().ctr_table_export(self._handle, replica, _np_ptr(keys), _np_ptr(x), _np_ptr(m),
                                    _np_ptr(v), _np_ptr(vhat), self.stream)
        if st != CTR_OK:
            raise RuntimeError("ctr_table_export: %d" % st)
        return {"keys": keys, "x": x, "m": m, "v": v, "vhat": vhat}

    def set_geometry(self, span=0, probe_items=0):
        """Test hook (ctr_debug_set_geometry); the workspace is grown for the larger probe tiles."""
        st = lib().ctr_debug_set_geometry(self._handle, span, probe_items)
        self._ws_slack = 1 << 20 if (span or probe_items) else 0
        return st

    def set_push_order(self, windows=0, split_launch=0, min_grad_bytes=256 << 20):
        """Measurement and test hook (ctr_debug_set_push_order)."""
        return lib().ctr_debug_set_push_order(self._handle, windows, split_launch, min_grad_bytes)

    def profile_enable(self, on=True):
        return lib().ctr_profile_enable(self._handle, 1 if on else 0)

    def profile_read(self):
        """{stage: (total ms, executions)} since the previous read."""
        ms = np.zeros(CTR_N_STAGES, np.float32)
        cnt = np.zeros(CTR_N_STAGES, np.uint32)
        st = lib().ctr_profile_read(self._handle, _np_ptr(ms), _np_ptr(cnt))
        if st != CTR_OK:
            raise RuntimeError("ctr_profile_read: %d" % st)
        return {n: (float(m), int(c)) for n, m, c in zip(STAGE_NAMES, ms, cnt)}
