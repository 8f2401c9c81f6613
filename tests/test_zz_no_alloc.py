"""The forward entry point that allocates nothing (`mgrit_fas_forward_static`: the library's own fixed
workspace instead of a workspace argument) against `mgrit_fas_forward`, through the C ABI.  Same kernels and
same schedule, so the outputs are compared bit for bit; two calls in a row, the second on a smaller problem
(the array keeps the first call's contents), plus the size limit."""
import ctypes

import numpy as np
import pytest

import mgrit_inputs as I

pytestmark = pytest.mark.gpu


def _run_both(wl, **overrides):
    import torch
    import paper_2007_07336_amd as M
    data = I.generate(wl)
    p = M.problem_from_workload(wl, **overrides)
    dev = "cuda:0"
    W = torch.from_numpy(data["W"]).to(dev)
    if wl.dtype == I.BF16:
        W = W.to(torch.bfloat16)
    b = torch.from_numpy(data["b"]).to(dev)
    u0 = torch.from_numpy(data["u0"]).to(dev)
    need = M.mgrit_workspace_bytes(p)
    assert 0 < need <= M.MGRIT_STATIC_SCRATCH_BYTES, need
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    U_ref = torch.zeros((wl.N + 1,) + wl.state_shape, dtype=torch.float32, device=dev)
    U_new = torch.full_like(U_ref, float("nan"))
    print(f"\n[case] {wl.name}: workspace {need} bytes, existing entry point", flush=True)
    rc, hist_ref, it_ref = M.mgrit_fas_forward(p, W, b, u0, U_ref, ws)
    torch.cuda.synchronize()
    print(f"[case] {wl.name}: static entry point", flush=True)
    before = torch.cuda.memory_allocated()
    rc2, hist_new, it_new = M.mgrit_fas_forward_static(p, W, b, u0, U_new)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert rc == rc2 == 0 and it_ref == it_new
    assert hist_ref == hist_new, (hist_ref, hist_new)
    assert torch.equal(U_ref, U_new)
    return U_new


def test_static_workspace_entry_point_matches_the_existing_one_twice_in_a_row():
    # first call: the benchmark's dense workload (32 MB of workspace: three levels, fused sweeps, norm partials)
    big = I.cfg2(2)
    _run_both(big)
    # second call right after it, smaller problem of a different kind, on the array the first call left behind
    small = I.reduced(I.cfg3(2), name="static_conv_c16_12x12_B3_N16", B=3, Himg=12, Wimg=12, N=16, m=4, act=I.TANH)
    _run_both(small)
    # and a run to a tolerance (host outputs, one synchronisation per cycle) with the RMS norm
    _run_both(I.reduced(I.cfg2(30), name="static_dense_q64_tol", q=64, B=20, N=64), tol=1e-6, norm_kind=1)


def test_static_workspace_entry_point_refuses_what_does_not_fit():
    import torch
    import paper_2007_07336_amd as M
    wl = I.cfg4(1)                                     # 1.9 GB of workspace
    p = M.problem_from_workload(wl)
    assert M.mgrit_workspace_bytes(p) > M.MGRIT_STATIC_SCRATCH_BYTES
    x = torch.zeros(64, dtype=torch.float32, device="cuda:0")     # never touched: the size check comes first
    rc, _, _ = M.mgrit_fas_forward_static(p, x, x, x, x, check=False)
    assert rc == M.binding.MGRIT_ERR_WORKSPACE
    bad = M.make_problem(N=16, h=1 / 16, m=1, max_levels=2, relax=0, max_iter=1, layer=0, act=0, dtype=0, B=4, q=8)
    rc, _, _ = M.mgrit_fas_forward_static(bad, x, x, x, x, check=False)
    assert rc == M.binding.MGRIT_ERR_PROBLEM
