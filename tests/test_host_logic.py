"""Host-side logic of the C-ABI library that needs no GPU: exported symbols, the level maps
(bit-exact against the oracle), workspace sizes and argument validation."""
import ctypes
import os
import re

import pytest

import mgrit_inputs as I
import paper_2007_07336_amd as M
from paper_2007_07336_amd import binding as Bd
from oracle import mgrit_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "mgrit.h")).read()
    names = set(re.findall(r"\b(mgrit_[a-z_]+)\s*\(", hdr))
    assert {"mgrit_level_map", "mgrit_workspace_bytes", "mgrit_adjoint_workspace_bytes", "mgrit_fas_forward",
            "mgrit_fas_adjoint", "mgrit_residual_norm"} <= names
    L = M.lib()
    for n in names:
        assert hasattr(L, n), n


def test_problem_struct_matches_header_field_order():
    hdr = open(os.path.join(ROOT, "include", "mgrit.h")).read()
    body = hdr[hdr.index("typedef struct mgrit_problem {"):hdr.index("} mgrit_problem_t;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in re.findall(r"(?:int32_t|float)\s+([^;]+);", body):
        fields += [f.strip() for f in decl.split(",")]
    assert fields == [f[0] for f in Bd.mgrit_problem_t._fields_]


def _problem(**kw):
    base = dict(N=16, h=1 / 16, m=4, max_levels=2, relax=0, max_iter=2, layer=0, act=0, dtype=0, B=4, q=8)
    base.update(kw)
    return M.make_problem(**base)


def test_level_maps_bit_exact_against_oracle():
    for m in (2, 3, 4, 8, 16):
        for N in list(range(1, 80)) + [256, 512, 1024, 4096]:
            for max_levels in (1, 2, 3, 6):
                for min_coarse in (0, 1, 8):
                    p = _problem(N=N, m=m, max_levels=max_levels, min_coarse=min_coarse)
                    try:
                        sizes_o, fidx_o = O.level_map(N, m, max_levels, min_coarse)
                    except ValueError:
                        with pytest.raises(M.MgritError) as e:
                            M.mgrit_level_map(p)
                        assert e.value.code == Bd.MGRIT_ERR_PROBLEM
                        continue
                    sizes, fidx = M.mgrit_level_map(p)
                    assert sizes == sizes_o
                    assert all(list(map(int, a)) == b for a, b in zip(fidx_o, fidx))


def test_benchmark_hierarchies():
    want = {"cfg1": [16, 4], "cfg2": [256, 64, 16], "cfg3": [64, 16], "cfg4": [512, 64, 8], "cfg5": [1024, 64, 4]}
    for k, f in I.ALL.items():
        assert M.mgrit_level_map(M.problem_from_workload(f()))[0] == want[k]


def test_workspace_sizes():
    p = M.problem_from_workload(I.cfg2())
    E = 128 * 256 * 4
    fwd = M.mgrit_workspace_bytes(p)
    # two coarse levels hold a state and a right-hand side per point, each fine level a C-point residual
    assert fwd >= (2 * 65 + 2 * 17 + 65 + 17) * E
    assert fwd < (2 * 65 + 2 * 17 + 65 + 17) * E + (1 << 20)
    # the adjoint adds the act' cache; a transposed copy of dense weights only when asked for
    adj = M.mgrit_adjoint_workspace_bytes(p)
    assert fwd + 256 * E <= adj < fwd + 256 * E + 4096
    os.environ["MGRIT_ADJ_TRANSPOSED"] = "1"
    try:
        adj_copy = M.mgrit_adjoint_workspace_bytes(p)
    finally:
        del os.environ["MGRIT_ADJ_TRANSPOSED"]
    assert 0 <= adj_copy - adj - 256 * 256 * 256 * 4 < 4096
    assert M.mgrit_workspace_bytes(_problem(m=1)) == 0
    assert M.mgrit_workspace_bytes(_problem(q=12)) == 0


# Non-null, 256-byte aligned and never dereferenced: every call below passes workspace_bytes = 0 (or 8),
# so even a problem that is valid is turned away with MGRIT_ERR_WORKSPACE before anything is launched.
FAKE = 1 << 20


def _fwd(p, W=FAKE, b=FAKE, u0=FAKE, U=FAKE, ws=FAKE, ws_bytes=0):
    return M.lib().mgrit_fas_forward(ctypes.byref(p), W, b, u0, U, None, None, ws, ws_bytes, None)


def test_forward_argument_validation():
    p = _problem()
    assert _fwd(p, W=None) == Bd.MGRIT_ERR_POINTER
    assert _fwd(p, U=None) == Bd.MGRIT_ERR_POINTER
    assert _fwd(p, u0=FAKE + 4) == Bd.MGRIT_ERR_POINTER              # misaligned
    assert _fwd(p, ws=None) == Bd.MGRIT_ERR_POINTER
    assert _fwd(p) == Bd.MGRIT_ERR_WORKSPACE
    assert _fwd(p, ws_bytes=M.mgrit_workspace_bytes(p) - 1) == Bd.MGRIT_ERR_WORKSPACE
    for bad in (dict(N=0), dict(m=1), dict(max_levels=0), dict(max_levels=17), dict(relax=2), dict(cycle=1),
                dict(max_iter=0), dict(norm_kind=2), dict(layer=2), dict(act=5), dict(dtype=3), dict(init=4), dict(init=-1),
                dict(h=0.0), dict(B=0), dict(q=0)):
        assert _fwd(_problem(**bad)) == Bd.MGRIT_ERR_PROBLEM, bad
    for ragged in (dict(N=18, m=4), dict(N=24, m=4, max_levels=3), dict(N=3, m=4)):   # level sizes that are no multiples of m are valid
        assert _fwd(_problem(**ragged)) == Bd.MGRIT_ERR_WORKSPACE, ragged
    assert M.mgrit_level_map(_problem(N=18, m=4))[0] == [18, 4]
    assert M.mgrit_level_map(_problem(N=24, m=4, max_levels=3))[0] == [24, 6, 1]
    assert M.mgrit_level_map(_problem(N=3, m=4))[0] == [3]
    for uns in (dict(q=12), dict(N=65536, m=2, max_levels=2), dict(layer=1, C=12, Himg=4, Wimg=4), dict(layer=1, C=128, Himg=4, Wimg=4),
                dict(layer=1, C=16, Himg=4, Wimg=300)):
        assert _fwd(_problem(**uns)) == Bd.MGRIT_ERR_UNSUPPORTED, uns
    assert _fwd(_problem(layer=1, C=0, Himg=4, Wimg=4)) == Bd.MGRIT_ERR_PROBLEM
    for ok_init in (Bd.MGRIT_INIT_ZERO, Bd.MGRIT_INIT_COPY, Bd.MGRIT_INIT_USER, Bd.MGRIT_INIT_NESTED):
        assert _fwd(_problem(init=ok_init)) == Bd.MGRIT_ERR_WORKSPACE     # valid problem: stops at the size check


def test_adjoint_and_norm_argument_validation():
    L = M.lib()
    p = _problem()
    rc = L.mgrit_fas_adjoint(ctypes.byref(p), FAKE, FAKE, FAKE, None, FAKE, None, None, None, None, FAKE, 0, None)
    assert rc == Bd.MGRIT_ERR_POINTER
    rc = L.mgrit_fas_adjoint(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, FAKE, None, None, None, None, FAKE, 8, None)
    assert rc == Bd.MGRIT_ERR_WORKSPACE
    rc = L.mgrit_residual_norm(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, None, FAKE, 0, None)
    assert rc == Bd.MGRIT_ERR_POINTER
    out = ctypes.c_double()
    rc = L.mgrit_residual_norm(ctypes.byref(p), FAKE, FAKE, FAKE, FAKE, ctypes.byref(out), FAKE, 8, None)
    assert rc == Bd.MGRIT_ERR_WORKSPACE
    rc = L.mgrit_level_map(None, None, None, None)
    assert rc == Bd.MGRIT_ERR_POINTER


def test_mixed_stack_argument_validation_and_workspace():
    L = M.lib()
    conv = _problem(layer=1, C=8, Himg=4, Wimg=4, q=0, N=16, m=2, max_levels=3)
    assert M.mgrit_workspace_bytes_mixed(conv, 4) >= M.mgrit_workspace_bytes(conv) > 0   # plus partials of the dense launches
    d, nfc = 4 * 4 * 8, 4
    # the fully connected matrices' adjoint runs on the caller's arrays: a transposed copy only when asked for
    extra = lambda: ((M.mgrit_adjoint_workspace_bytes_mixed(conv, 4) - M.mgrit_workspace_bytes_mixed(conv, 4))
                     - (M.mgrit_adjoint_workspace_bytes(conv) - M.mgrit_workspace_bytes(conv)))
    assert extra() == 0
    os.environ["MGRIT_ADJ_TRANSPOSED"] = "1"
    try:
        assert extra() >= nfc * d * d * 4
    finally:
        del os.environ["MGRIT_ADJ_TRANSPOSED"]
    assert M.mgrit_workspace_bytes_mixed(conv, 1) == 0 and M.mgrit_workspace_bytes_mixed(conv, 0) == 0
    assert M.mgrit_workspace_bytes_mixed(_problem(), 4) == 0                               # dense stacks have no mixed form
    big = _problem(layer=1, C=64, Himg=32, Wimg=32, q=0)                                   # d = 65536: d*d overflows
    assert M.mgrit_workspace_bytes_mixed(big, 4) == 0
    fc = Bd.mgrit_fc_layers_t(fc_period=4, Wfc=FAKE, bfc=FAKE, dWfc=None, dbfc=None)
    rc = L.mgrit_fas_forward_mixed(ctypes.byref(conv), None, FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 1 << 40, None)
    assert rc == Bd.MGRIT_ERR_POINTER
    rc = L.mgrit_fas_forward_mixed(ctypes.byref(conv), ctypes.byref(fc), FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 8, None)
    assert rc == Bd.MGRIT_ERR_WORKSPACE
    nofc = Bd.mgrit_fc_layers_t(fc_period=4, Wfc=None, bfc=FAKE, dWfc=None, dbfc=None)
    rc = L.mgrit_fas_forward_mixed(ctypes.byref(conv), ctypes.byref(nofc), FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 8, None)
    assert rc == Bd.MGRIT_ERR_POINTER
    for bad_period in (1, -3):
        bad = Bd.mgrit_fc_layers_t(fc_period=bad_period, Wfc=FAKE, bfc=FAKE, dWfc=None, dbfc=None)
        rc = L.mgrit_fas_forward_mixed(ctypes.byref(conv), ctypes.byref(bad), FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 8, None)
        assert rc == Bd.MGRIT_ERR_PROBLEM
    zero = Bd.mgrit_fc_layers_t(fc_period=0, Wfc=FAKE, bfc=FAKE, dWfc=None, dbfc=None)
    rc = L.mgrit_fas_forward_mixed(ctypes.byref(conv), ctypes.byref(zero), FAKE, FAKE, FAKE, FAKE, None, None, FAKE, 8, None)
    assert rc == Bd.MGRIT_ERR_PROBLEM
    # the adjoint wants dWfc with dW (and dbfc with db)
    rc = L.mgrit_fas_adjoint_mixed(ctypes.byref(conv), ctypes.byref(fc), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, None,
                                   FAKE, 8, None)
    assert rc == Bd.MGRIT_ERR_POINTER
    rc = L.mgrit_fas_adjoint_mixed(ctypes.byref(conv), ctypes.byref(fc), FAKE, FAKE, FAKE, FAKE, FAKE, None, None, None, None,
                                   FAKE, 8, None)
    assert rc == Bd.MGRIT_ERR_WORKSPACE
    out = ctypes.c_double()
    rc = L.mgrit_residual_norm_mixed(ctypes.byref(conv), ctypes.byref(fc), FAKE, FAKE, FAKE, FAKE, ctypes.byref(out), FAKE, 8, None)
    assert rc == Bd.MGRIT_ERR_WORKSPACE


def test_fc_layers_struct_matches_header_field_order():
    hdr = open(os.path.join(ROOT, "include", "mgrit.h")).read()
    body = hdr[hdr.index("typedef struct mgrit_fc_layers {"):hdr.index("} mgrit_fc_layers_t;")]
    fields = re.findall(r"([A-Za-z_]+);", body)
    assert fields == [f[0] for f in Bd.mgrit_fc_layers_t._fields_]


def test_inputs_are_reproducible_and_bf16_exact():
    import numpy as np
    wl = I.reduced(I.cfg5(1), q=16, B=3, N=4, m=2)
    a, b = I.generate(wl), I.generate(wl)
    assert all(np.array_equal(a[k], b[k]) for k in a)
    W = a["W"]
    assert np.array_equal(W.view(np.uint32) & 0xFFFF, np.zeros(W.shape, np.uint32))
    x = np.array([1.0, 1.00390625, 1.005859375, -1.01171875, 3.0e38], np.float32)
    # ties to even: 1 + 2^-8 (exact tie between 1 and 1 + 2^-7) rounds to 1
    assert list(I.round_to_bf16(x)[:2]) == [1.0, 1.0]
    import torch
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(I.round_to_bf16(x), ref)


def test_static_workspace_entry_point_checks_size_and_problem_before_touching_the_gpu():
    """mgrit_fas_forward_static refuses a problem whose workspace exceeds the library's fixed array, and an invalid
    problem, from host logic alone (no GPU call is made before these checks)."""
    big = M.make_problem(N=512, h=1 / 512, m=8, max_levels=3, relax=1, max_iter=1, layer=1, act=1, dtype=1, B=32,
                         C=64, Himg=32, Wimg=32)
    assert M.mgrit_workspace_bytes(big) > M.MGRIT_STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(256)
    L = M.lib()
    assert L.mgrit_fas_forward_static(ctypes.byref(big), fake, fake, fake, fake, None, None, None) == Bd.MGRIT_ERR_WORKSPACE
    bad = _problem(m=1)
    assert L.mgrit_fas_forward_static(ctypes.byref(bad), fake, fake, fake, fake, None, None, None) == Bd.MGRIT_ERR_PROBLEM
    assert L.mgrit_fas_forward_static(None, fake, fake, fake, fake, None, None, None) == Bd.MGRIT_ERR_POINTER
    hdr = open(os.path.join(ROOT, "include", "mgrit.h")).read()
    assert "MGRIT_STATIC_SCRATCH_BYTES = 64 * 1024 * 1024" in hdr and M.MGRIT_STATIC_SCRATCH_BYTES == 64 * 1024 * 1024


def test_bench_reads_measured_traffic_from_the_profile_tables():
    import bench
    v = bench.measured_traffic_bytes("cfg2", "dense_sweep_kernel<float>")
    assert v is not None and 5e7 < v < 2e8                      # fetch + write of one 64-interval sweep, bytes
    assert bench.measured_traffic_bytes("no_such_workload", "dense_sweep_kernel<float>") is None
    with pytest.raises(RuntimeError):                           # a table that does not list the kernel is stale
        bench.measured_traffic_bytes("cfg2", "conv_sweep_kernel")
    for cls in Bd.TRACE_CLASSES:                                # every traced step-kernel class has a row pattern
        if cls != "dense_grad_kernel":
            assert cls in bench.PROFILE_ROW, cls
