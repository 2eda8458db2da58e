"""ctypes binding of libidkm.so: the same entry points as include/idkm.h, argument marshalling only.

PyTorch supplies device memory and the current HIP stream; every step of the
method runs inside the library's kernels.  There is no CPU fallback: if the
shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("IDKM_LIB", os.path.join(HERE, "libidkm.so"))

IDKM_OK = 0
STATUS_NAMES = {0: "IDKM_OK", 1: "IDKM_ERR_INVALID_ARG", 2: "IDKM_ERR_ALLOC", 3: "IDKM_ERR_DEVICE",
                4: "IDKM_ERR_NONFINITE", 5: "IDKM_ERR_NO_FORWARD", 6: "IDKM_ERR_UNSUPPORTED"}
DIST_L2, DIST_SQL2 = 0, 1
BWD_IMPLICIT, BWD_JFB, BWD_DENSE, BWD_GMRES = 0, 1, 2, 3
PATH_AUTO, PATH_STREAM, PATH_PERSISTENT = 0, 1, 2

EXPORTS = ["idkm_version", "idkm_limits", "idkm_status_string", "idkm_create", "idkm_destroy", "idkm_last_error",
           "idkm_set_path", "idkm_set_matrix_cores", "idkm_set_tile_limit", "idkm_set_spin_limit", "idkm_set_kernel_timing", "idkm_last_kernel_ms", "idkm_set_gmres_basis", "idkm_advance_sequence", "idkm_forward", "idkm_backward", "idkm_step_F", "idkm_step_JCT", "idkm_get_cotangents", "idkm_forward_noalloc", "idkm_noalloc_last_error",
           "idkm_calibrate", "idkm_code_bits", "idkm_code_words", "idkm_pack_codes", "idkm_unpack_quantize",
           "idkm_batch_create", "idkm_batch_destroy", "idkm_batch_last_error", "idkm_batch_launches",
           "idkm_batch_context", "idkm_batch_forward", "idkm_batch_backward"]


class IdkmInfo(C.Structure):
    _fields_ = [("iters", C.c_int32), ("converged", C.c_int32), ("residual", C.c_double),
                ("empty_clusters", C.c_int32), ("path", C.c_int32), ("alpha", C.c_double)]


class IdkmFwdDesc(C.Structure):
    _fields_ = [("W", C.c_void_p), ("m", C.c_int64), ("d", C.c_int32), ("C0", C.c_void_p), ("k", C.c_int32),
                ("tau", C.c_float), ("tol", C.c_float), ("max_iter", C.c_int32), ("dist", C.c_int32),
                ("C_out", C.c_void_p), ("A_out", C.c_void_p), ("Wq_out", C.c_void_p), ("assign_out", C.c_void_p)]


class IdkmBwdDesc(C.Structure):
    _fields_ = [("dWq", C.c_void_p), ("mode", C.c_int32), ("tol", C.c_float), ("max_iter", C.c_int32),
                ("alpha", C.c_float), ("dW_out", C.c_void_p)]


class IdkmLimits(C.Structure):
    _fields_ = [("max_k", C.c_int32), ("max_d", C.c_int32), ("max_kd", C.c_int32)]


class IdkmError(RuntimeError):
    def __init__(self, status: int, detail: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {detail}")
        self.status = status
        self.detail = detail


_lib = None


def load_library():
    """dlopen libidkm.so (built in-tree by paper_2312_07759_amd.build).  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2312_07759_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, f32p, i32p = C.c_void_p, C.c_void_p, C.c_void_p
    lib.idkm_version.restype = C.c_int32
    lib.idkm_limits.argtypes = [C.POINTER(IdkmLimits)]
    lib.idkm_limits.restype = None
    lib.idkm_status_string.argtypes = [C.c_int]
    lib.idkm_status_string.restype = C.c_char_p
    lib.idkm_create.argtypes = [C.POINTER(vp), C.c_int]
    lib.idkm_create.restype = C.c_int
    lib.idkm_destroy.argtypes = [vp]
    lib.idkm_destroy.restype = C.c_int
    lib.idkm_last_error.argtypes = [vp]
    lib.idkm_last_error.restype = C.c_char_p
    lib.idkm_set_path.argtypes = [vp, C.c_int]
    lib.idkm_set_path.restype = C.c_int
    lib.idkm_set_tile_limit.argtypes = [vp, C.c_int64]
    lib.idkm_set_tile_limit.restype = C.c_int
    lib.idkm_set_matrix_cores.argtypes = [vp, C.c_int32]
    lib.idkm_set_matrix_cores.restype = C.c_int
    lib.idkm_set_spin_limit.argtypes = [vp, C.c_uint32]
    lib.idkm_set_spin_limit.restype = C.c_int
    lib.idkm_set_kernel_timing.argtypes = [vp, C.c_int32]
    lib.idkm_set_kernel_timing.restype = C.c_int
    lib.idkm_last_kernel_ms.argtypes = [vp, C.POINTER(C.c_float)]
    lib.idkm_last_kernel_ms.restype = C.c_int
    lib.idkm_advance_sequence.argtypes = [vp, C.c_uint32, vp]
    lib.idkm_advance_sequence.restype = C.c_int
    lib.idkm_set_gmres_basis.argtypes = [vp, C.c_int32]
    lib.idkm_set_gmres_basis.restype = C.c_int
    lib.idkm_forward.argtypes = [vp, f32p, C.c_int64, C.c_int32, f32p, C.c_int32, C.c_float, C.c_float, C.c_int32,
                                 C.c_int, f32p, f32p, f32p, i32p, C.POINTER(IdkmInfo), vp]
    lib.idkm_forward.restype = C.c_int
    lib.idkm_backward.argtypes = [vp, f32p, C.c_int, C.c_float, C.c_int32, C.c_float, f32p, C.POINTER(IdkmInfo), vp]
    lib.idkm_backward.restype = C.c_int
    lib.idkm_step_F.argtypes = [vp, f32p, C.c_int64, C.c_int32, f32p, C.c_int32, C.c_float, C.c_int, f32p, f32p, vp]
    lib.idkm_step_F.restype = C.c_int
    lib.idkm_step_JCT.argtypes = [vp, f32p, f32p, vp]
    lib.idkm_step_JCT.restype = C.c_int
    lib.idkm_forward_noalloc.argtypes = [C.c_int, f32p, C.c_int64, C.c_int32, f32p, C.c_int32, C.c_float, C.c_float,
                                         C.c_int32, C.c_int, f32p, f32p, f32p, i32p, C.POINTER(IdkmInfo), vp]
    lib.idkm_forward_noalloc.restype = C.c_int
    lib.idkm_noalloc_last_error.argtypes = []
    lib.idkm_noalloc_last_error.restype = C.c_char_p
    lib.idkm_get_cotangents.argtypes = [vp, vp, vp, vp]
    lib.idkm_get_cotangents.restype = C.c_int
    lib.idkm_calibrate.argtypes = [vp, C.c_int32, f32p, C.c_int64, C.POINTER(C.c_double), vp]
    lib.idkm_calibrate.restype = C.c_int
    lib.idkm_code_bits.argtypes = [C.c_int32]
    lib.idkm_code_bits.restype = C.c_int32
    lib.idkm_code_words.argtypes = [C.c_int64, C.c_int32]
    lib.idkm_code_words.restype = C.c_int64
    lib.idkm_pack_codes.argtypes = [vp, i32p, C.c_int64, C.c_int32, vp, vp]
    lib.idkm_pack_codes.restype = C.c_int
    lib.idkm_unpack_quantize.argtypes = [vp, vp, C.c_int64, f32p, C.c_int32, C.c_int32, f32p, vp]
    lib.idkm_unpack_quantize.restype = C.c_int
    lib.idkm_batch_create.argtypes = [C.POINTER(vp), C.c_int, C.c_int32]
    lib.idkm_batch_create.restype = C.c_int
    lib.idkm_batch_destroy.argtypes = [vp]
    lib.idkm_batch_destroy.restype = C.c_int
    lib.idkm_batch_last_error.argtypes = [vp]
    lib.idkm_batch_last_error.restype = C.c_char_p
    lib.idkm_batch_launches.argtypes = [vp]
    lib.idkm_batch_launches.restype = C.c_int32
    lib.idkm_batch_context.argtypes = [vp, C.c_int32]
    lib.idkm_batch_context.restype = vp
    lib.idkm_batch_forward.argtypes = [vp, C.POINTER(IdkmFwdDesc), C.c_int32, C.POINTER(IdkmInfo), C.POINTER(C.c_int), vp]
    lib.idkm_batch_forward.restype = C.c_int
    lib.idkm_batch_backward.argtypes = [vp, C.POINTER(IdkmBwdDesc), C.c_int32, C.POINTER(IdkmInfo), C.POINTER(C.c_int), vp]
    lib.idkm_batch_backward.restype = C.c_int
    _lib = lib
    return lib


@dataclass
class Info:
    iters: int
    converged: bool
    residual: float
    empty_clusters: int
    path: int
    alpha: float


def _info(i: IdkmInfo) -> Info:
    return Info(int(i.iters), bool(i.converged), float(i.residual), int(i.empty_clusters), int(i.path), float(i.alpha))


def _ptr(t, dtype, shape, name):
    """Device pointer of a contiguous torch tensor after checking dtype/shape/device."""
    import torch
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a tensor in device memory")
    if t.dtype != dtype or not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise TypeError(f"{name} must be contiguous {dtype} of shape {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")
    return C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Context:
    """Owns an idkm_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, device: int = 0):
        self._lib = load_library()
        h = C.c_void_p()
        st = self._lib.idkm_create(C.byref(h), int(device))
        if st != IDKM_OK:
            raise IdkmError(st, "idkm_create failed")
        self._h = h
        self.device = int(device)
        self._keep = None

    def close(self):
        if getattr(self, "_h", None):
            self._lib.idkm_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st):
        if st != IDKM_OK:
            raise IdkmError(st, self._lib.idkm_last_error(self._h).decode())

    def set_path(self, path: int):
        self._check(self._lib.idkm_set_path(self._h, int(path)))

    def set_tile_limit(self, nbytes: int):
        self._check(self._lib.idkm_set_tile_limit(self._h, int(nbytes)))

    def set_matrix_cores(self, enable: bool):
        self._check(self._lib.idkm_set_matrix_cores(self._h, 1 if enable else 0))

    def advance_sequence(self, n: int):
        self._check(self._lib.idkm_advance_sequence(self._h, int(n), _stream()))

    def set_gmres_basis(self, basis: int):
        self._check(self._lib.idkm_set_gmres_basis(self._h, int(basis)))

    def set_kernel_timing(self, enable: bool):
        self._check(self._lib.idkm_set_kernel_timing(self._h, 1 if enable else 0))

    def last_kernel_ms(self) -> float:
        """idkm_last_kernel_ms: event time of the last persistent launch (needs set_kernel_timing(True))."""
        ms = C.c_float()
        self._check(self._lib.idkm_last_kernel_ms(self._h, C.byref(ms)))
        return float(ms.value)

    def set_spin_limit(self, polls: int):
        self._check(self._lib.idkm_set_spin_limit(self._h, int(polls)))

    def forward(self, W, C0, tau, tol, max_iter, dist, want_A=False, want_Wq=True, want_assign=False, out=None):
        """idkm_forward.  W [m,d], C0 [k,d] float32 device tensors.  Returns dict(C, A, Wq, assign, info).
        `out` may hold preallocated tensors under the keys C, A, Wq, assign (as a training loop would keep them)."""
        import torch
        m, d = W.shape
        k = C0.shape[0]
        dev = W.device
        out = out or {}
        Cout = out.get("C")
        if Cout is None:
            Cout = torch.empty((k, d), dtype=torch.float32, device=dev)
        A = out.get("A") if want_A else None
        if want_A and A is None:
            A = torch.empty((m, k), dtype=torch.float32, device=dev)
        Wq = out.get("Wq") if want_Wq else None
        if want_Wq and Wq is None:
            Wq = torch.empty((m, d), dtype=torch.float32, device=dev)
        asg = out.get("assign") if want_assign else None
        if want_assign and asg is None:
            asg = torch.empty((m,), dtype=torch.int32, device=dev)
        info = IdkmInfo()
        st = self._lib.idkm_forward(self._h, _ptr(W, torch.float32, (m, d), "W"), m, d,
                                    _ptr(C0, torch.float32, (k, d), "C0"), k, float(tau), float(tol), int(max_iter),
                                    int(dist), _ptr(Cout, torch.float32, (k, d), "C_out"),
                                    _ptr(A, torch.float32, (m, k), "A_out"), _ptr(Wq, torch.float32, (m, d), "Wq_out"),
                                    _ptr(asg, torch.int32, (m,), "assign_out"), C.byref(info), _stream())
        self._check(st)
        self._keep = W  # the library borrows W until backward
        return dict(C=Cout, A=A, Wq=Wq, assign=asg, info=_info(info))

    def backward(self, dWq, mode, tol=1e-6, max_iter=1000, alpha=1.0, out=None):
        """idkm_backward.  dWq [m,d] float32 device tensor.  Returns dict(dW, info); `out` may be a preallocated dW."""
        import torch
        dW = out if out is not None else torch.empty_like(dWq)
        info = IdkmInfo()
        st = self._lib.idkm_backward(self._h, _ptr(dWq, torch.float32, dWq.shape, "dWq"), int(mode), float(tol),
                                     int(max_iter), float(alpha), _ptr(dW, torch.float32, dWq.shape, "dW_out"),
                                     C.byref(info), _stream())
        self._check(st)
        return dict(dW=dW, info=_info(info))

    def get_cotangents(self, k, d):
        """idkm_get_cotangents: (v, g) of the last backward as float64 numpy arrays [k,d]."""
        import numpy as np
        v = np.empty((k, d), dtype=np.float64)
        g = np.empty((k, d), dtype=np.float64)
        self._check(self._lib.idkm_get_cotangents(self._h, v.ctypes.data_as(C.c_void_p), g.ctypes.data_as(C.c_void_p),
                                                  _stream()))
        return v, g

    def calibrate(self, kind, buf=None):
        """idkm_calibrate: 0 lane-ops/s, 1 exponentials/s, 2 bytes/s of a streaming read of `buf` (float32 tensor),
        3-5 exponentials/s beside 1, 2, 4 FMAs, 6-8 float32 matrix multiply-adds/s (16x16x4, 16x16x4 with vector FMAs
        between, 4x4x1)."""
        import torch
        r = C.c_double()
        n = 0 if buf is None else buf.numel()
        ptr = None if buf is None else _ptr(buf, torch.float32, buf.shape, "buf")
        self._check(self._lib.idkm_calibrate(self._h, int(kind), ptr, n, C.byref(r), _stream()))
        return float(r.value)

    def pack_codes(self, assign, k):
        """idkm_pack_codes: int32 [m] device tensor -> int32 tensor holding the uint32 words of the b-bit stream."""
        import torch
        m = assign.shape[0]
        words = torch.empty((max(code_words(m, k), 0),), dtype=torch.int32, device=assign.device)
        st = self._lib.idkm_pack_codes(self._h, _ptr(assign, torch.int32, (m,), "assign"), m, int(k),
                                       C.c_void_p(words.data_ptr()), _stream())
        self._check(st)
        return words

    def unpack_quantize(self, words, m, Cb):
        """idkm_unpack_quantize: stream words + codebook [k,d] -> q(W, C) [m,d]."""
        import torch
        k, d = Cb.shape
        out = torch.empty((m, d), dtype=torch.float32, device=Cb.device)
        st = self._lib.idkm_unpack_quantize(self._h, _ptr(words, torch.int32, (code_words(m, k),), "words"), m,
                                            _ptr(Cb, torch.float32, (k, d), "C"), k, d,
                                            _ptr(out, torch.float32, (m, d), "Wh_out"), _stream())
        self._check(st)
        return out

    def step_F(self, W, Cb, tau, dist):
        """idkm_step_F: one evaluation of F at Cb.  Returns (C+ [k,d], n [k])."""
        import torch
        m, d = W.shape
        k = Cb.shape[0]
        Cp = torch.empty((k, d), dtype=torch.float32, device=W.device)
        n = torch.empty((k,), dtype=torch.float32, device=W.device)
        st = self._lib.idkm_step_F(self._h, _ptr(W, torch.float32, (m, d), "W"), m, d,
                                   _ptr(Cb, torch.float32, (k, d), "C"), k, float(tau), int(dist),
                                   _ptr(Cp, torch.float32, (k, d), "Cplus_out"), _ptr(n, torch.float32, (k,), "n_out"),
                                   _stream())
        self._check(st)
        self._keep = W
        return Cp, n

    def step_JCT(self, g):
        """idkm_step_JCT: (dF/dC)^T g at the state left by step_F / forward."""
        import torch
        out = torch.empty_like(g)
        st = self._lib.idkm_step_JCT(self._h, _ptr(g, torch.float32, g.shape, "g"),
                                     _ptr(out, torch.float32, g.shape, "out"), _stream())
        self._check(st)
        return out


def forward_noalloc(W, C0, tau, tol, max_iter, dist, out, device: int = 0, want_info: bool = True):
    """idkm_forward_noalloc.  `out` holds the caller's preallocated device tensors: C [k,d] (required) and
    optionally A [m,k], Wq [m,d], assign int32 [m].  Returns Info, or None when want_info is False (then the solve
    is only enqueued on the current stream)."""
    import torch
    lib = load_library()
    m, d = W.shape
    k = C0.shape[0]
    info = IdkmInfo()
    st = lib.idkm_forward_noalloc(int(device), _ptr(W, torch.float32, (m, d), "W"), m, d,
                                  _ptr(C0, torch.float32, (k, d), "C0"), k, float(tau), float(tol), int(max_iter),
                                  int(dist), _ptr(out["C"], torch.float32, (k, d), "C_out"),
                                  _ptr(out.get("A"), torch.float32, (m, k), "A_out"),
                                  _ptr(out.get("Wq"), torch.float32, (m, d), "Wq_out"),
                                  _ptr(out.get("assign"), torch.int32, (m,), "assign_out"),
                                  C.byref(info) if want_info else None, _stream())
    if st != IDKM_OK:
        raise IdkmError(st, lib.idkm_noalloc_last_error().decode())
    return _info(info) if want_info else None


def code_bits(k: int) -> int:
    return int(load_library().idkm_code_bits(int(k)))


def code_words(m: int, k: int) -> int:
    return int(load_library().idkm_code_words(int(m), int(k)))


class Batch:
    """Owns an idkm_batch: one context per layer; forward/backward over all layers in as few launches as fit."""

    def __init__(self, n_layers: int, device: int = 0):
        self._lib = load_library()
        h = C.c_void_p()
        st = self._lib.idkm_batch_create(C.byref(h), int(device), int(n_layers))
        if st != IDKM_OK:
            raise IdkmError(st, "idkm_batch_create failed")
        self._h = h
        self.n_layers = int(n_layers)
        self._keep = None

    def close(self):
        if getattr(self, "_h", None):
            self._lib.idkm_batch_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def launches(self) -> int:
        return int(self._lib.idkm_batch_launches(self._h))

    def set_path(self, path: int):
        for i in range(self.n_layers):
            st = self._lib.idkm_set_path(self._lib.idkm_batch_context(self._h, i), int(path))
            if st != IDKM_OK:
                raise IdkmError(st, "idkm_set_path failed")

    def context_set_spin_limit(self, i: int, polls: int):
        """idkm_set_spin_limit on the i-th layer's context."""
        st = self._lib.idkm_set_spin_limit(self._lib.idkm_batch_context(self._h, int(i)), int(polls))
        if st != IDKM_OK:
            raise IdkmError(st, "idkm_set_spin_limit failed")

    def _finish(self, st, statuses, strict):
        if st != IDKM_OK and strict:
            raise IdkmError(st, self._lib.idkm_batch_last_error(self._h).decode())
        return [int(x) for x in statuses]

    def forward(self, layers, tau, tol, max_iter, dist, want_Wq=True, want_assign=False, strict=True):
        """idkm_batch_forward.  layers: list of (W [m,d], C0 [k,d]) float32 device tensors (shapes may differ);
        tau may be a scalar or one value per layer.  Returns a list of dict(C, Wq, assign, info, status)."""
        import torch
        n = len(layers)
        taus = list(tau) if hasattr(tau, "__len__") else [tau] * n
        descs = (IdkmFwdDesc * n)()
        infos = (IdkmInfo * n)()
        statuses = (C.c_int * n)()
        outs = []
        for i, (W, C0) in enumerate(layers):
            m, d = W.shape
            k = C0.shape[0]
            Cout = torch.empty((k, d), dtype=torch.float32, device=W.device)
            Wq = torch.empty((m, d), dtype=torch.float32, device=W.device) if want_Wq else None
            asg = torch.empty((m,), dtype=torch.int32, device=W.device) if want_assign else None
            descs[i] = IdkmFwdDesc(_ptr(W, torch.float32, (m, d), "W"), m, d, _ptr(C0, torch.float32, (k, d), "C0"), k,
                                   float(taus[i]), float(tol), int(max_iter), int(dist),
                                   _ptr(Cout, torch.float32, (k, d), "C_out"), None,
                                   _ptr(Wq, torch.float32, (m, d), "Wq_out"), _ptr(asg, torch.int32, (m,), "assign_out"))
            outs.append(dict(C=Cout, Wq=Wq, assign=asg))
        st = self._lib.idkm_batch_forward(self._h, descs, n, infos, statuses, _stream())
        sts = self._finish(st, statuses, strict)
        self._keep = [W for W, _ in layers]  # the library borrows every W until the backward
        for i, o in enumerate(outs):
            o["info"] = _info(infos[i])
            o["status"] = sts[i]
        return outs

    def backward(self, dWqs, mode, tol=1e-6, max_iter=1000, alpha=1.0, strict=True):
        """idkm_batch_backward.  dWqs: one [m,d] float32 device tensor per layer.  Returns list of dict(dW, info, status)."""
        import torch
        n = len(dWqs)
        descs = (IdkmBwdDesc * n)()
        infos = (IdkmInfo * n)()
        statuses = (C.c_int * n)()
        outs = []
        for i, g in enumerate(dWqs):
            dW = torch.empty_like(g)
            descs[i] = IdkmBwdDesc(_ptr(g, torch.float32, g.shape, "dWq"), int(mode), float(tol), int(max_iter),
                                   float(alpha), _ptr(dW, torch.float32, g.shape, "dW_out"))
            outs.append(dict(dW=dW))
        st = self._lib.idkm_batch_backward(self._h, descs, n, infos, statuses, _stream())
        sts = self._finish(st, statuses, strict)
        for i, o in enumerate(outs):
            o["info"] = _info(infos[i])
            o["status"] = sts[i]
        return outs


def limits():
    lib = load_library()
    lim = IdkmLimits()
    lib.idkm_limits(C.byref(lim))
    return dict(max_k=lim.max_k, max_d=lim.max_d, max_kd=lim.max_kd)
