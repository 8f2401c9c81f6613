"""Helpers for the GPU parity tests: run a workload through the C-ABI library and through the
CPU oracle on the same seeded inputs."""
from __future__ import annotations

import numpy as np

import mgrit_inputs as I
from oracle import mgrit_oracle as O


def rel_l2_per_state(got: np.ndarray, ref: np.ndarray) -> float:
    """max over the leading (point / layer) axis of ||got - ref|| / ||ref||."""
    g = got.reshape(got.shape[0], -1).astype(np.float64)
    r = ref.reshape(ref.shape[0], -1).astype(np.float64)
    num = np.linalg.norm(g - r, axis=1)
    den = np.linalg.norm(r, axis=1)
    den = np.where(den > 0, den, 1.0)
    return float((num / den).max())


def to_dev(x: np.ndarray, bf16: bool = False):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda")
    if bf16:
        t = t.to(torch.bfloat16)          # exact: the values are bf16-representable already
    return t


class GpuProblem:
    """Device buffers of one workload."""

    def __init__(self, wl: I.Workload, data: dict, **problem_overrides):
        import torch
        import paper_2007_07336_amd as M
        self.M = M
        self.wl = wl
        self.p = M.problem_from_workload(wl, **problem_overrides)
        self.W = to_dev(data["W"], wl.dtype == I.BF16)
        self.b = to_dev(data["b"])
        self.u0 = to_dev(data["u0"])
        self.U = torch.zeros((wl.N + 1,) + wl.state_shape, dtype=torch.float32, device="cuda")
        nbytes = max(M.mgrit_workspace_bytes(self.p), 256)
        assert M.mgrit_workspace_bytes(self.p) > 0
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")

    def forward(self, U_init=None, check=True):
        import torch
        if U_init is not None:
            self.U.copy_(torch.from_numpy(np.ascontiguousarray(U_init, dtype=np.float32)))
        rc, hist, it = self.M.mgrit_fas_forward(self.p, self.W, self.b, self.u0, self.U, self.ws, check=check)
        torch.cuda.synchronize()
        return rc, self.U.cpu().numpy(), hist, it

    def residual_norm(self, U: np.ndarray):
        import torch
        Ud = to_dev(U.astype(np.float32))
        rc, v = self.M.mgrit_residual_norm(self.p, self.W, self.b, self.u0, Ud, self.ws)
        return v

    def adjoint(self, U: np.ndarray, lamN: np.ndarray, want_grad=True, Lam_init=None):
        import torch
        M, wl = self.M, self.wl
        nbytes = M.mgrit_adjoint_workspace_bytes(self.p)
        assert nbytes > 0
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        Ud = to_dev(U.astype(np.float32))
        lam = to_dev(lamN.astype(np.float32))
        Lam = torch.zeros_like(Ud)
        if Lam_init is not None:
            Lam.copy_(torch.from_numpy(np.ascontiguousarray(Lam_init, dtype=np.float32)))
        dW = torch.zeros(self.W.shape, dtype=torch.float32, device="cuda") if want_grad else None
        db = torch.zeros_like(self.b) if want_grad else None
        rc, hist, it = M.mgrit_fas_adjoint(self.p, self.W, self.b, Ud, lam, Lam, dW, db, ws)
        torch.cuda.synchronize()
        return (Lam.cpu().numpy(), None if dW is None else dW.cpu().numpy(),
                None if db is None else db.cpu().numpy(), hist, it)


def oracle_forward(wl: I.Workload, data: dict, init=1, U_init=None, max_iter=None, tol=None, norm_kind=None):
    return O.fas_forward(data["W"], data["b"], data["u0"], wl.h, wl.m, wl.max_levels, wl.min_coarse, wl.relax,
                         wl.max_iter if max_iter is None else max_iter, wl.layer, wl.act,
                         tol=wl.tol if tol is None else tol,
                         norm_kind=wl.norm_kind if norm_kind is None else norm_kind, init=init, U_init=U_init)


def oracle_adjoint(wl: I.Workload, data: dict, U, lamN, init=1, Lam_init=None):
    return O.fas_adjoint(data["W"], data["b"], U, lamN, wl.h, wl.m, wl.max_levels, wl.min_coarse, wl.relax,
                         wl.max_iter, wl.layer, wl.act, tol=wl.tol, norm_kind=wl.norm_kind, init=init,
                         Lam_init=Lam_init)
