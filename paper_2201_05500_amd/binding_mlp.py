"""ctypes binding of the dense-tower C ABI (include/ctr_mlp.h): marshalling only."""
from __future__ import annotations

import ctypes as C

import numpy as np

from .binding import CTR_OK, CTR_STEP_LOCAL, lib as _base_lib

CTR_MLP_MAX_HIDDEN = 6
EXPORTED = ("ctr_mlp_bytes", "ctr_mlp_workspace_bytes", "ctr_mlp_create", "ctr_mlp_destroy", "ctr_mlp_step",
            "ctr_mlp_forward", "ctr_mlp_step_bf16", "ctr_mlp_step_bf16_grad_bf16", "ctr_mlp_forward_bf16", "ctr_mlp_gemm", "ctr_mlp_kstep_merge", "ctr_mlp_n_params", "ctr_mlp_export", "ctr_mlp_import")


class ctr_mlp_config(C.Structure):
    _fields_ = [
        ("in_dim", C.c_uint32),
        ("n_hidden", C.c_uint32),
        ("hidden", C.c_uint32 * CTR_MLP_MAX_HIDDEN),
        ("n_replicas", C.c_uint32),
        ("kstep", C.c_uint32),
        ("lr", C.c_float),
        ("beta1", C.c_float),
        ("beta2", C.c_float),
        ("eps", C.c_float),
        ("init_seed", C.c_uint64),
    ]


_ready = False


def lib():
    global _ready
    L = _base_lib()
    if not _ready:
        vp, u32, sz, ci = C.c_void_p, C.c_uint32, C.c_size_t, C.c_int
        cfgp = C.POINTER(ctr_mlp_config)
        L.ctr_mlp_bytes.restype = sz
        L.ctr_mlp_bytes.argtypes = [cfgp]
        L.ctr_mlp_n_params.restype = sz
        L.ctr_mlp_n_params.argtypes = [cfgp]
        L.ctr_mlp_workspace_bytes.restype = sz
        L.ctr_mlp_workspace_bytes.argtypes = [cfgp, u32]
        L.ctr_mlp_create.restype = ci
        L.ctr_mlp_create.argtypes = [cfgp, vp, sz, vp, C.POINTER(vp)]
        L.ctr_mlp_destroy.restype = ci
        L.ctr_mlp_destroy.argtypes = [vp]
        L.ctr_mlp_step.restype = ci
        L.ctr_mlp_step.argtypes = [vp, u32, vp, vp, u32, vp, vp, vp, sz, u32, vp]
        L.ctr_mlp_forward.restype = ci
        L.ctr_mlp_forward.argtypes = [vp, u32, vp, u32, vp, vp, sz, vp]
        L.ctr_mlp_step_bf16.restype = ci
        L.ctr_mlp_step_bf16.argtypes = L.ctr_mlp_step.argtypes
        L.ctr_mlp_step_bf16_grad_bf16.restype = ci
        L.ctr_mlp_step_bf16_grad_bf16.argtypes = L.ctr_mlp_step.argtypes
        L.ctr_mlp_forward_bf16.restype = ci
        L.ctr_mlp_forward_bf16.argtypes = L.ctr_mlp_forward.argtypes
        L.ctr_mlp_gemm.restype = ci
        L.ctr_mlp_gemm.argtypes = [ci, ci, vp, u32, vp, u32, u32, u32, u32, vp, u32, vp, sz, vp]
        L.ctr_mlp_kstep_merge.restype = ci
        L.ctr_mlp_kstep_merge.argtypes = [vp, vp]
        L.ctr_mlp_export.restype = ci
        L.ctr_mlp_export.argtypes = [vp, u32, vp, vp, vp, vp, vp]
        L.ctr_mlp_import.restype = ci
        L.ctr_mlp_import.argtypes = [vp, u32, vp, vp, vp, vp, u32, vp]
        _ready = True
    return L


def make_config(in_dim, hidden, n_replicas=1, kstep=False, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, init_seed=0):
    h = (C.c_uint32 * CTR_MLP_MAX_HIDDEN)(*([int(x) for x in hidden] + [0] * (CTR_MLP_MAX_HIDDEN - len(hidden))))
    return ctr_mlp_config(in_dim, len(hidden), h, n_replicas, 1 if kstep else 0, lr, beta1, beta2, eps, init_seed)


class CtrMlp:
    """Owns the torch allocations of one tower and forwards to the ABI."""

    def __init__(self, in_dim, hidden, n_replicas=1, kstep=False, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8,
                 init_seed=0, device="cuda:0"):
        import torch
        self._torch = torch
        self.device = torch.device(device)
        if len(hidden) > CTR_MLP_MAX_HIDDEN:
            raise ValueError("too many hidden layers")
        self.cfg = make_config(in_dim, hidden, n_replicas, kstep, lr, beta1, beta2, eps, init_seed)
        self.in_dim, self.kstep, self.W = int(in_dim), bool(kstep), int(n_replicas)
        nbytes = int(lib().ctr_mlp_bytes(C.byref(self.cfg)))
        if nbytes == 0:
            raise ValueError("invalid tower configuration")
        self.n_params = int(lib().ctr_mlp_n_params(C.byref(self.cfg)))
        self._mem = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self._ws, self.ws_bytes, self._handle = None, 0, None
        out = C.c_void_p()
        st = lib().ctr_mlp_create(C.byref(self.cfg), self._mem.data_ptr(), nbytes, self.stream, C.byref(out))
        if st != CTR_OK:
            raise RuntimeError("ctr_mlp_create failed: %d" % st)
        self._handle = out.value

    @property
    def stream(self) -> int:
        return int(self._torch.cuda.current_stream(self.device).cuda_stream)

    def reserve(self, batch):
        need = int(lib().ctr_mlp_workspace_bytes(C.byref(self.cfg), batch))
        if need == 0:
            raise ValueError("invalid batch")
        if need > self.ws_bytes:
            self._torch.cuda.synchronize(self.device)
            self._ws = self._torch.empty(need, dtype=self._torch.uint8, device=self.device)
            self.ws_bytes = need

    def close(self):
        if self._handle:
            self._torch.cuda.synchronize(self.device)
            lib().ctr_mlp_destroy(self._handle)
            self._handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step(self, replica, pooled, labels, grad_pooled=None, mode=CTR_STEP_LOCAL, loss=None):
        """pooled f32 or bf16 [B, in], labels f32 [B] (device).  Returns (status, loss tensor[1], grad_pooled):
        the gradient is fp32 unless a bfloat16 `grad_pooled` is passed in (bf16 input only)."""
        torch = self._torch
        B = pooled.shape[0]
        self.reserve(B)
        if grad_pooled is None:
            grad_pooled = torch.empty(pooled.shape, dtype=torch.float32, device=self.device)
        if loss is None:
            loss = torch.empty(1, dtype=torch.float32, device=self.device)
        if grad_pooled.dtype == torch.bfloat16:
            if pooled.dtype != torch.bfloat16:
                raise ValueError("a bfloat16 gradient needs a bfloat16 input")
            fn = lib().ctr_mlp_step_bf16_grad_bf16
        else:
            fn = lib().ctr_mlp_step_bf16 if pooled.dtype == torch.bfloat16 else lib().ctr_mlp_step
        st = fn(self._handle, replica, pooled.data_ptr(), labels.data_ptr(), B, grad_pooled.data_ptr(),
                loss.data_ptr(), self._ws.data_ptr(), self.ws_bytes, mode, self.stream)
        return st, loss, grad_pooled

    def forward(self, replica, pooled):
        torch = self._torch
        B = pooled.shape[0]
        self.reserve(B)
        logits = torch.empty(B, dtype=torch.float32, device=self.device)
        fn = lib().ctr_mlp_forward_bf16 if pooled.dtype == torch.bfloat16 else lib().ctr_mlp_forward
        st = fn(self._handle, replica, pooled.data_ptr(), B, logits.data_ptr(), self._ws.data_ptr(), self.ws_bytes,
                self.stream)
        return st, logits

    def kstep_merge(self):
        return lib().ctr_mlp_kstep_merge(self._handle, self.stream)

    def load(self, replica=0, params=None, m=None, v=None, vhat=None, pending=False):
        """Restores state exported earlier (float32 numpy arrays of n_params elements; None = keep)."""
        arrs = [None if a is None else np.ascontiguousarray(a, dtype=np.float32) for a in (params, m, v, vhat)]
        for a in arrs:
            if a is not None and a.size != self.n_params:
                raise ValueError("wrong length")
        ptr = lambda a: None if a is None else a.ctypes.data_as(C.c_void_p)
        return lib().ctr_mlp_import(self._handle, replica, ptr(arrs[0]), ptr(arrs[1]), ptr(arrs[2]), ptr(arrs[3]),
                                    1 if pending else 0, self.stream)

    def export(self, replica=0):
        n = self.n_params
        p, m, v = (np.empty(n, np.float32) for _ in range(3))
        vh = np.empty(n, np.float32) if self.kstep else None
        ptr = lambda a: None if a is None else a.ctypes.data_as(C.c_void_p)
        st = lib().ctr_mlp_export(self._handle, replica, ptr(p), ptr(m), ptr(v), ptr(vh), self.stream)
        if st != CTR_OK:
            raise RuntimeError("ctr_mlp_export: %d" % st)
        return {"params": p, "m": m, "v": v, "vhat": vh}


def ctr_mlp_gemm(a_k_contiguous, b_k_contiguous, d_a, lda, d_b, ldb, m, n, k, d_c, ldc, d_scratch, scratch_bytes,
                 stream) -> int:
    return lib().ctr_mlp_gemm(1 if a_k_contiguous else 0, 1 if b_k_contiguous else 0, d_a, lda, d_b, ldb, m, n, k, d_c,
                              ldc, d_scratch, scratch_bytes, stream)
