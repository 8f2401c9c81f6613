"""ctypes binding of libmgrit.so.  Argument marshalling only: every step of the method runs
in the library's HIP kernels.  torch is used for device memory and the current stream.

The functions carry the names of the C entry points declared in include/mgrit.h.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmgrit.so")

MGRIT_OK = 0
MGRIT_ERR_POINTER, MGRIT_ERR_PROBLEM, MGRIT_ERR_WORKSPACE = -1, -2, -3
MGRIT_ERR_UNSUPPORTED, MGRIT_ERR_NONFINITE, MGRIT_ERR_HIP = -4, -5, -6
MGRIT_MAX_LEVELS = 16
MGRIT_INIT_ZERO, MGRIT_INIT_COPY, MGRIT_INIT_USER, MGRIT_INIT_NESTED = 0, 1, 2, 3
ERROR_NAMES = {0: "MGRIT_OK", -1: "MGRIT_ERR_POINTER", -2: "MGRIT_ERR_PROBLEM", -3: "MGRIT_ERR_WORKSPACE",
               -4: "MGRIT_ERR_UNSUPPORTED", -5: "MGRIT_ERR_NONFINITE", -6: "MGRIT_ERR_HIP"}


class MgritError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where} returned {ERROR_NAMES.get(code, code)}")
        self.code = code


class mgrit_problem_t(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("h", ctypes.c_float), ("m", ctypes.c_int32),
                ("max_levels", ctypes.c_int32), ("min_coarse", ctypes.c_int32), ("relax", ctypes.c_int32),
                ("cycle", ctypes.c_int32), ("max_iter", ctypes.c_int32), ("tol", ctypes.c_float),
                ("norm_kind", ctypes.c_int32), ("layer", ctypes.c_int32), ("act", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("B", ctypes.c_int32), ("q", ctypes.c_int32),
                ("C", ctypes.c_int32), ("Himg", ctypes.c_int32), ("Wimg", ctypes.c_int32),
                ("init", ctypes.c_int32)]


class mgrit_fc_layers_t(ctypes.Structure):
    _fields_ = [("fc_period", ctypes.c_int32), ("Wfc", ctypes.c_void_p), ("bfc", ctypes.c_void_p),
                ("dWfc", ctypes.c_void_p), ("dbfc", ctypes.c_void_p)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2007_07336_amd.build` "
                               "(or __graft_entry__.build()) first; there is no CPU fallback")
        L = ctypes.CDLL(LIB_PATH)
        P = ctypes.POINTER(mgrit_problem_t)
        vp, i32p, dp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)
        L.mgrit_level_map.argtypes = [P, i32p, i32p, i32p]
        L.mgrit_level_map.restype = ctypes.c_int32
        L.mgrit_workspace_bytes.argtypes = [P]
        L.mgrit_workspace_bytes.restype = ctypes.c_size_t
        L.mgrit_adjoint_workspace_bytes.argtypes = [P]
        L.mgrit_adjoint_workspace_bytes.restype = ctypes.c_size_t
        L.mgrit_fas_forward.argtypes = [P, vp, vp, vp, vp, dp, i32p, vp, ctypes.c_size_t, vp]
        L.mgrit_fas_forward.restype = ctypes.c_int32
        L.mgrit_fas_forward_static.argtypes = [P, vp, vp, vp, vp, dp, i32p, vp]
        L.mgrit_fas_forward_static.restype = ctypes.c_int32
        L.mgrit_fas_adjoint.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, dp, i32p, vp, ctypes.c_size_t, vp]
        L.mgrit_fas_adjoint.restype = ctypes.c_int32
        L.mgrit_residual_norm.argtypes = [P, vp, vp, vp, vp, dp, vp, ctypes.c_size_t, vp]
        L.mgrit_residual_norm.restype = ctypes.c_int32
        F = ctypes.POINTER(mgrit_fc_layers_t)
        L.mgrit_workspace_bytes_mixed.argtypes = [P, ctypes.c_int32]
        L.mgrit_workspace_bytes_mixed.restype = ctypes.c_size_t
        L.mgrit_adjoint_workspace_bytes_mixed.argtypes = [P, ctypes.c_int32]
        L.mgrit_adjoint_workspace_bytes_mixed.restype = ctypes.c_size_t
        L.mgrit_fas_forward_mixed.argtypes = [P, F, vp, vp, vp, vp, dp, i32p, vp, ctypes.c_size_t, vp]
        L.mgrit_fas_forward_mixed.restype = ctypes.c_int32
        L.mgrit_fas_adjoint_mixed.argtypes = [P, F, vp, vp, vp, vp, vp, vp, vp, dp, i32p, vp, ctypes.c_size_t, vp]
        L.mgrit_fas_adjoint_mixed.restype = ctypes.c_int32
        L.mgrit_residual_norm_mixed.argtypes = [P, F, vp, vp, vp, vp, dp, vp, ctypes.c_size_t, vp]
        L.mgrit_residual_norm_mixed.restype = ctypes.c_int32
        L.mgrit_trace_begin.argtypes = []
        L.mgrit_trace_begin.restype = None
        L.mgrit_trace_end.argtypes = [dp, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64), dp,
                                      ctypes.c_int32]
        L.mgrit_trace_end.restype = ctypes.c_int32
        _lib = L
    return _lib


def make_problem(*, N, h, m, max_levels, relax, max_iter, layer, act, dtype, B, q=0, C=0, Himg=0, Wimg=0,
                 min_coarse=1, tol=0.0, norm_kind=0, init=1, cycle=0) -> mgrit_problem_t:
    return mgrit_problem_t(N=N, h=h, m=m, max_levels=max_levels, min_coarse=min_coarse, relax=relax, cycle=cycle,
                           max_iter=max_iter, tol=tol, norm_kind=norm_kind, layer=layer, act=act, dtype=dtype,
                           B=B, q=q, C=C, Himg=Himg, Wimg=Wimg, init=init)


def problem_from_workload(wl, **overrides) -> mgrit_problem_t:
    """Problem struct from a workload description (fields N, m, ... as in mgrit_inputs.Workload)."""
    kw = dict(N=wl.N, h=wl.h, m=wl.m, max_levels=wl.max_levels, relax=wl.relax, max_iter=wl.max_iter,
              layer=wl.layer, act=wl.act, dtype=wl.dtype, B=wl.B, q=wl.q, C=wl.C, Himg=wl.Himg, Wimg=wl.Wimg,
              min_coarse=wl.min_coarse, tol=wl.tol, norm_kind=wl.norm_kind)
    kw.update(overrides)
    return make_problem(**kw)


def mgrit_level_map(p: mgrit_problem_t):
    """Returns (N_l list, fine_index list of lists); raises MgritError on an invalid hierarchy."""
    L = lib()
    n = ctypes.c_int32(0)
    Nl = (ctypes.c_int32 * MGRIT_MAX_LEVELS)()
    rc = L.mgrit_level_map(ctypes.byref(p), ctypes.byref(n), Nl, None)
    if rc != MGRIT_OK:
        raise MgritError(rc, "mgrit_level_map")
    sizes = [Nl[i] for i in range(n.value)]
    total = sum(s + 1 for s in sizes)
    fi = (ctypes.c_int32 * total)()
    rc = L.mgrit_level_map(ctypes.byref(p), ctypes.byref(n), Nl, fi)
    if rc != MGRIT_OK:
        raise MgritError(rc, "mgrit_level_map")
    out, pos = [], 0
    for s in sizes:
        out.append([fi[pos + j] for j in range(s + 1)])
        pos += s + 1
    return sizes, out


def mgrit_workspace_bytes(p: mgrit_problem_t) -> int:
    return int(lib().mgrit_workspace_bytes(ctypes.byref(p)))


def mgrit_adjoint_workspace_bytes(p: mgrit_problem_t) -> int:
    return int(lib().mgrit_adjoint_workspace_bytes(ctypes.byref(p)))


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def mgrit_fas_forward(p: mgrit_problem_t, W, b, u0, U, workspace, *, want_hist=True, stream=None,
                      check=True):
    """Enqueues the forward solve.  Tensors are CUDA(HIP) tensors owned by the caller.
    Returns (return code, residual history list, cycles done)."""
    hist = (ctypes.c_double * max(p.max_iter, 1))() if want_hist else None
    iters = ctypes.c_int32(0)
    rc = lib().mgrit_fas_forward(ctypes.byref(p), _ptr(W), _ptr(b), _ptr(u0), _ptr(U), hist,
                                 ctypes.byref(iters) if want_hist else None, _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream))
    if check and rc != MGRIT_OK:
        raise MgritError(rc, "mgrit_fas_forward")
    return rc, ([hist[i] for i in range(iters.value)] if want_hist else None), iters.value


MGRIT_STATIC_SCRATCH_BYTES = 64 * 1024 * 1024


def mgrit_fas_forward_static(p: mgrit_problem_t, W, b, u0, U, *, want_hist=True, stream=None, check=True):
    """mgrit_fas_forward on the library's own fixed workspace (no workspace argument, nothing allocated)."""
    hist = (ctypes.c_double * max(p.max_iter, 1))() if want_hist else None
    iters = ctypes.c_int32(0)
    rc = lib().mgrit_fas_forward_static(ctypes.byref(p), _ptr(W), _ptr(b), _ptr(u0), _ptr(U), hist,
                                        ctypes.byref(iters) if want_hist else None, _stream(stream))
    if check and rc != MGRIT_OK:
        raise MgritError(rc, "mgrit_fas_forward_static")
    return rc, ([hist[i] for i in range(iters.value)] if want_hist else None), iters.value


def mgrit_fas_adjoint(p: mgrit_problem_t, W, b, U, lamN, Lam, dW, db, workspace, *, want_hist=True,
                      stream=None, check=True):
    hist = (ctypes.c_double * max(p.max_iter, 1))() if want_hist else None
    iters = ctypes.c_int32(0)
    rc = lib().mgrit_fas_adjoint(ctypes.byref(p), _ptr(W), _ptr(b), _ptr(U), _ptr(lamN), _ptr(Lam), _ptr(dW),
                                 _ptr(db), hist, ctypes.byref(iters) if want_hist else None, _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream))
    if check and rc != MGRIT_OK:
        raise MgritError(rc, "mgrit_fas_adjoint")
    return rc, ([hist[i] for i in range(iters.value)] if want_hist else None), iters.value


def mgrit_residual_norm(p: mgrit_problem_t, W, b, u0, U, workspace, *, stream=None, check=True):
    out = ctypes.c_double(0.0)
    rc = lib().mgrit_residual_norm(ctypes.byref(p), _ptr(W), _ptr(b), _ptr(u0), _ptr(U), ctypes.byref(out),
                                   _ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream(stream))
    if check and rc != MGRIT_OK:
        raise MgritError(rc, "mgrit_residual_norm")
    return rc, out.value


def make_fc_layers(fc_period: int, Wfc, bfc, dWfc=None, dbfc=None) -> mgrit_fc_layers_t:
    """Fully connected layers of a mixed stack (device tensors owned by the caller, which keeps them alive)."""
    return mgrit_fc_layers_t(fc_period=fc_period, Wfc=_ptr(Wfc), bfc=_ptr(bfc), dWfc=_ptr(dWfc), dbfc=_ptr(dbfc))


def mgrit_workspace_bytes_mixed(p: mgrit_problem_t, fc_period: int) -> int:
    return int(lib().mgrit_workspace_bytes_mixed(ctypes.byref(p), fc_period))


def mgrit_adjoint_workspace_bytes_mixed(p: mgrit_problem_t, fc_period: int) -> int:
    return int(lib().mgrit_adjoint_workspace_bytes_mixed(ctypes.byref(p), fc_period))


def mgrit_fas_forward_mixed(p: mgrit_problem_t, fc: mgrit_fc_layers_t, W, b, u0, U, workspace, *, want_hist=True,
                            stream=None, check=True):
    hist = (ctypes.c_double * max(p.max_iter, 1))() if want_hist else None
    iters = ctypes.c_int32(0)
    rc = lib().mgrit_fas_forward_mixed(ctypes.byref(p), ctypes.byref(fc), _ptr(W), _ptr(b), _ptr(u0), _ptr(U), hist,
                                       ctypes.byref(iters) if want_hist else None, _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream))
    if check and rc != MGRIT_OK:
        raise MgritError(rc, "mgrit_fas_forward_mixed")
    return rc, ([hist[i] for i in range(iters.value)] if want_hist else None), iters.value


def mgrit_fas_adjoint_mixed(p: mgrit_problem_t, fc: mgrit_fc_layers_t, W, b, U, lamN, Lam, dW, db, workspace, *,
                            want_hist=True, stream=None, check=True):
    hist = (ctypes.c_double * max(p.max_iter, 1))() if want_hist else None
    iters = ctypes.c_int32(0)
    rc = lib().mgrit_fas_adjoint_mixed(ctypes.byref(p), ctypes.byref(fc), _ptr(W), _ptr(b), _ptr(U), _ptr(lamN),
                                       _ptr(Lam), _ptr(dW), _ptr(db), hist,
                                       ctypes.byref(iters) if want_hist else None, _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream))
    if check and rc != MGRIT_OK:
        raise MgritError(rc, "mgrit_fas_adjoint_mixed")
    return rc, ([hist[i] for i in range(iters.value)] if want_hist else None), iters.value


def mgrit_residual_norm_mixed(p: mgrit_problem_t, fc: mgrit_fc_layers_t, W, b, u0, U, workspace, *, stream=None,
                              check=True):
    out = ctypes.c_double(0.0)
    rc = lib().mgrit_residual_norm_mixed(ctypes.byref(p), ctypes.byref(fc), _ptr(W), _ptr(b), _ptr(u0), _ptr(U),
                                         ctypes.byref(out), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream))
    if check and rc != MGRIT_OK:
        raise MgritError(rc, "mgrit_residual_norm_mixed")
    return rc, out.value


TRACE_CLASSES = ("dense_step_kernel<float,64,64>", "dense_step_kernel<float,128,128>",
                 "dense_step_kernel<bf16,64,64>", "dense_step_kernel<bf16,128,128>",
                 "conv_step_kernel<float>", "conv_step_kernel<bf16>", "dense_grad_kernel",
                 "dense_sweep_kernel<float>", "dense_sweep_kernel<bf16>", "dense_ksplit_kernel<float,8>",
                 "dense_ksplit_kernel<float,4>", "dense_ksplit_kernel<bf16,4>", "dense_ksplit_kernel<bf16,8>",
                 "conv_sweep_kernel")


def mgrit_trace_begin() -> None:
    lib().mgrit_trace_begin()


def mgrit_trace_end() -> dict:
    """{kernel class: (total ms, launches, layer steps, algorithmic bytes)} of the launches since
    mgrit_trace_begin()."""
    n = len(TRACE_CLASSES)
    ms = (ctypes.c_double * n)()
    la = (ctypes.c_int64 * n)()
    un = (ctypes.c_int64 * n)()
    by = (ctypes.c_double * n)()
    rc = lib().mgrit_trace_end(ms, la, un, by, n)
    if rc != MGRIT_OK:
        raise MgritError(rc, "mgrit_trace_end")
    return {TRACE_CLASSES[i]: (ms[i], la[i], un[i], by[i]) for i in range(n) if la[i] > 0}
