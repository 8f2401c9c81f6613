"""GPU parity of stacks that mix convolution layers with periodic fully connected layers (Sec. IV-E):
the HIP path through the C ABI against the CPU oracle on the same seeded inputs, element by element."""
import numpy as np
import pytest

import mgrit_inputs as I
from oracle import mgrit_oracle as O
from tests.gpu_util import rel_l2_per_state, to_dev

pytestmark = pytest.mark.gpu

TOL = {I.FP32: 1e-5, I.BF16: 2e-2}      # relative L2 per state / per layer gradient


def _announce(name):
    print(f"\n[case] {name}", flush=True)


class GpuMixed:
    """Device buffers of one mixed workload."""

    def __init__(self, wl, data, **overrides):
        import torch
        import paper_2007_07336_amd as M
        self.M, self.wl = M, wl
        self.p = M.problem_from_workload(wl, **overrides)
        bf = wl.dtype == I.BF16
        self.W, self.b, self.u0 = to_dev(data["W"], bf), to_dev(data["b"]), to_dev(data["u0"])
        self.Wfc, self.bfc = to_dev(data["Wfc"], bf), to_dev(data["bfc"])
        self.U = torch.zeros((wl.N + 1,) + wl.state_shape, dtype=torch.float32, device="cuda")
        n = M.mgrit_workspace_bytes_mixed(self.p, wl.fc_period)
        assert n > 0
        self.ws = torch.empty(n, dtype=torch.uint8, device="cuda")
        self.fc = M.make_fc_layers(wl.fc_period, self.Wfc, self.bfc)

    def forward(self):
        import torch
        rc, hist, it = self.M.mgrit_fas_forward_mixed(self.p, self.fc, self.W, self.b, self.u0, self.U, self.ws)
        torch.cuda.synchronize()
        return self.U.cpu().numpy(), hist, it

    def residual_norm(self, U):
        Ud = to_dev(U.astype(np.float32))
        return self.M.mgrit_residual_norm_mixed(self.p, self.fc, self.W, self.b, self.u0, Ud, self.ws)[1]

    def adjoint(self, U, lamN):
        import torch
        M, wl = self.M, self.wl
        ws = torch.empty(M.mgrit_adjoint_workspace_bytes_mixed(self.p, wl.fc_period), dtype=torch.uint8, device="cuda")
        Ud, lam = to_dev(U.astype(np.float32)), to_dev(lamN.astype(np.float32))
        Lam = torch.zeros_like(Ud)
        # outputs start from a sentinel: every entry, the zero slots included, must be written
        dW = torch.full(self.W.shape, 7.0, dtype=torch.float32, device="cuda")
        db = torch.full(self.b.shape, 7.0, dtype=torch.float32, device="cuda")
        dWfc = torch.full(self.Wfc.shape, 7.0, dtype=torch.float32, device="cuda")
        dbfc = torch.full(self.bfc.shape, 7.0, dtype=torch.float32, device="cuda")
        fc = M.make_fc_layers(wl.fc_period, self.Wfc, self.bfc, dWfc, dbfc)
        rc, hist, it = M.mgrit_fas_adjoint_mixed(self.p, fc, self.W, self.b, Ud, lam, Lam, dW, db, ws)
        torch.cuda.synchronize()
        return [t.cpu().numpy() for t in (Lam, dW, db, dWfc, dbfc)] + [hist, it]


def _oracle_forward(wl, data, init=1):
    Ws, bs, kinds = I.per_layer_lists(wl, data)
    return O.fas_forward(Ws, bs, data["u0"], wl.h, wl.m, wl.max_levels, wl.min_coarse, wl.relax, wl.max_iter,
                         kinds, wl.act, init=init)


def _mx(name, **kw):
    base = dict(name=name, B=3, C=16, Himg=6, Wimg=5, N=16, m=2, max_levels=3, fc_period=4, max_iter=2)
    base.update(kw)
    return I.reduced(I.mixed(2), **base)


MIXED_CASES = [
    # fully connected layers on C-points of every level (period a multiple of m^(L-1))
    _mx("mixed_fp32_c16_6x5_N16_m2_L3_P4"),
    # period not aligned with the coarsening: fully connected layers also on F-points, irregular per launch
    _mx("mixed_fp32_c8_5x4_N18_m3_L2_P5", C=8, Himg=5, Wimg=4, B=2, N=18, m=3, max_levels=2, fc_period=5),
    # only layer 0 is fully connected; F-relaxation
    _mx("mixed_fp32_c8_4x4_N8_P64_F", C=8, Himg=4, Wimg=4, N=8, fc_period=64, relax=I.RELAX_F),
    # every other layer fully connected
    _mx("mixed_fp32_c8_4x4_N8_P2", C=8, Himg=4, Wimg=4, N=8, fc_period=2),
    # serial propagation (one level): single-group launches that are wholly one kind or the other
    _mx("mixed_fp32_c16_4x4_N6_serial_P3", Himg=4, Wimg=4, N=6, max_levels=1, fc_period=3, max_iter=1),
    # bf16, 64 channels (the wide convolution tile), tanh
    _mx("mixed_bf16_c64_4x4_N16_m4_L2_P8", dtype=I.BF16, C=64, Himg=4, Wimg=4, B=2, m=4, max_levels=2, fc_period=8,
        act=I.TANH),
    # d = 2048: the dense launches of the fully connected groups use the tiled kernels, not only the small-launch one
    _mx("mixed_fp32_c32_8x8_N16_m2_L2_P2_d2048", C=32, Himg=8, Wimg=8, B=40, N=16, max_levels=2, fc_period=2, max_iter=1),
    # at most 32 samples: the fully connected steps take the k-split kernel (skinny launch) (d = 2048 float, 4096 bf16)
    _mx("mixed_fp32_c32_8x8_B20_N8_P2_d2048_deep_ksplit", C=32, Himg=8, Wimg=8, B=20, N=8, max_levels=2, fc_period=2, max_iter=1),
    _mx("mixed_bf16_c64_8x8_B8_N4_P2_d4096_deep_ksplit", dtype=I.BF16, C=64, Himg=8, Wimg=8, B=8, N=4, max_levels=2, fc_period=2,
        max_iter=1, act=I.TANH),
    # level sizes that are no multiples of m (23 -> 7 -> 2): trailing F-points of both kinds of layer
    _mx("mixed_fp32_c8_5x4_N23_m3_L3_P4_trailing", C=8, Himg=5, Wimg=4, B=2, N=23, m=3, fc_period=4),
]


@pytest.mark.parametrize("wl", MIXED_CASES, ids=lambda w: w.name)
def test_mixed_forward(wl):
    _announce(wl.name)
    data = I.generate(wl)
    gp = GpuMixed(wl, data)
    U, hist, it = gp.forward()
    Uo, hist_o, it_o = _oracle_forward(wl, data)
    assert rel_l2_per_state(U, Uo) <= TOL[wl.dtype]
    assert it == it_o
    for a, b in zip(hist, hist_o):
        assert abs(a - b) <= (1e-3 if wl.dtype == I.FP32 else 5e-2) * max(b, 1e-6)
    # the residual entry point, on states far enough from a solution that the residual is not rounding noise
    # (with bf16 operands the residual of the path's own solution is its rounding, not the oracle's)
    Ws, bs, kinds = I.per_layer_lists(wl, data)
    Up = (Uo + 0.05 * np.random.default_rng(5).standard_normal(Uo.shape)).astype(np.float32)
    r = gp.residual_norm(Up)
    ro = O.residual_norm(Ws, bs, data["u0"], Up.astype(np.float64), wl.h, kinds, wl.act)
    assert abs(r - ro) <= (1e-4 if wl.dtype == I.FP32 else 2e-2) * ro


def test_mixed_nested_start_and_serial_limit():
    wl = _mx("mixed_fp32_nested_P4", max_iter=8, relax=I.RELAX_F, max_levels=2, m=2)
    _announce(wl.name)
    data = I.generate(wl)
    gp = GpuMixed(wl, data, init=3)
    U, hist, it = gp.forward()
    Uo, hist_o, _ = _oracle_forward(wl, data, init=3)
    assert rel_l2_per_state(U, Uo) <= 1e-5
    # two-level F-relaxation is exact after N/m cycles: the serial propagation through both kinds of layer
    Ws, bs, kinds = I.per_layer_lists(wl, data)
    Us = O.serial_forward(Ws, bs, data["u0"], wl.h, kinds, wl.act)
    assert rel_l2_per_state(U, Us) <= 1e-5


MIXED_ADJ_CASES = [
    _mx("mixed_adj_fp32_c16_6x5_N16_m2_L3_P4", act=I.TANH),
    _mx("mixed_adj_fp32_c8_5x4_N18_m3_L2_P5", C=8, Himg=5, Wimg=4, B=2, N=18, m=3, max_levels=2, fc_period=5, act=I.TANH),
    _mx("mixed_adj_fp32_c8_4x4_N8_P2_F", C=8, Himg=4, Wimg=4, N=8, fc_period=2, relax=I.RELAX_F, act=I.TANH),
    _mx("mixed_adj_bf16_c64_4x4_N16_m4_L2_P8_relu", dtype=I.BF16, C=64, Himg=4, Wimg=4, B=2, m=4, max_levels=2,
        fc_period=8),
    _mx("mixed_adj_fp32_c32_8x8_N16_P2_d2048", C=32, Himg=8, Wimg=8, B=40, N=16, max_levels=2, fc_period=2, max_iter=1,
        act=I.TANH),
    _mx("mixed_adj_fp32_c32_8x8_B20_N8_P2_d2048_deep_ksplit", C=32, Himg=8, Wimg=8, B=20, N=8, max_levels=2, fc_period=2, max_iter=1,
        act=I.TANH),
    _mx("mixed_adj_fp32_c8_5x4_N23_m3_L3_P4_trailing", C=8, Himg=5, Wimg=4, B=2, N=23, m=3, fc_period=4, act=I.TANH),
]


@pytest.mark.parametrize("wl", MIXED_ADJ_CASES, ids=lambda w: w.name)
def test_mixed_adjoint_and_gradient(wl):
    _announce(wl.name)
    data = I.generate(wl)
    Ws, bs, kinds = I.per_layer_lists(wl, data)
    Uo, _, _ = _oracle_forward(wl, data)
    U = Uo.astype(np.float32)
    if wl.dtype == I.BF16 and wl.act == I.RELU:
        U = I.round_to_bf16(U)      # both sides take the ReLU' decision on the same bf16 operand
    lamN = np.random.default_rng(9).standard_normal(wl.state_shape).astype(np.float32)
    gp = GpuMixed(wl, data)
    Lam, dW, db, dWfc, dbfc, hist, it = gp.adjoint(U, lamN)
    Lo, dWo, dbo, hist_o, it_o = O.fas_adjoint(Ws, bs, U, lamN, wl.h, wl.m, wl.max_levels, wl.min_coarse, wl.relax,
                                               wl.max_iter, kinds, wl.act)
    tol = TOL[wl.dtype]
    assert it == it_o
    assert rel_l2_per_state(Lam, Lo) <= tol
    P = wl.fc_period
    for n in range(wl.N):
        if n % P == 0:
            k = n // P
            assert not dW[n].any() and not db[n].any()            # convolution slots of fully connected layers: zero
            eW, eb = rel_l2_per_state(dWfc[k][None], dWo[n][None]), rel_l2_per_state(dbfc[k][None], dbo[n][None])
        else:
            eW, eb = rel_l2_per_state(dW[n][None], dWo[n][None]), rel_l2_per_state(db[n][None], dbo[n][None])
        assert eW <= tol and eb <= tol, (n, eW, eb)


AS_STORED_MIXED = [w for w in MIXED_CASES if w.name in (
    "mixed_fp32_c16_6x5_N16_m2_L3_P4", "mixed_bf16_c64_4x4_N16_m4_L2_P8", "mixed_fp32_c32_8x8_N16_m2_L2_P2_d2048",
    "mixed_fp32_c32_8x8_B20_N8_P2_d2048_deep_ksplit", "mixed_bf16_c64_8x8_B8_N4_P2_d4096_deep_ksplit")]


@pytest.mark.parametrize("wl", AS_STORED_MIXED, ids=lambda w: w.name)
def test_mixed_adjoint_fc_weights_as_stored_and_transposed_copy(wl, monkeypatch):
    """The fully connected layers' adjoint reads the caller's matrices as stored; MGRIT_ADJ_TRANSPOSED=1 runs it on
    transposed copies in the workspace instead.  Same arithmetic in the same order: equal bit for bit."""
    _announce(wl.name)
    data = I.generate(wl)
    gp = GpuMixed(wl, data)
    U, _, _ = gp.forward()
    if wl.dtype == I.BF16 and wl.act == I.RELU:
        U = I.round_to_bf16(U)
    lamN = np.random.default_rng(9).standard_normal(wl.state_shape).astype(np.float32)
    n_default = gp.M.mgrit_adjoint_workspace_bytes_mixed(gp.p, wl.fc_period)
    res = gp.adjoint(U, lamN)
    monkeypatch.setenv("MGRIT_ADJ_TRANSPOSED", "1")
    n_copy = gp.M.mgrit_adjoint_workspace_bytes_mixed(gp.p, wl.fc_period)
    ref = gp.adjoint(U, lamN)
    monkeypatch.delenv("MGRIT_ADJ_TRANSPOSED")
    assert n_copy - n_default >= data["Wfc"].size * (4 if wl.dtype == I.FP32 else 2)
    for x, y in zip(res[:5], ref[:5]):
        assert np.array_equal(x, y)
    assert res[5] == ref[5] and res[6] == ref[6]


# ------------------------------------------------------------------ the benchmark's mixed workload at full size
def test_mixed_full_size_forward_elementwise():
    wl = I.mixed(2)
    _announce(wl.name)
    data = I.generate(wl)
    gp = GpuMixed(wl, data)
    U, hist, it = gp.forward()
    Uo, hist_o, _ = _oracle_forward(wl, data)
    err = rel_l2_per_state(U, Uo)
    print(f"mixed forward: {err:.3e}  residuals {hist} vs {hist_o}", flush=True)
    assert err <= 1e-5, err
    for a, b in zip(hist, hist_o):
        assert abs(a - b) <= 1e-3 * b


def test_mixed_full_size_adjoint_elementwise():
    """ReLU' is a 0/1 decision on the sign of z, so both sides must see the same z: weights (steps of 2^-7 below
    1/2), biases (steps of 2^-12) and the states to linearise about (steps of 2^-5 below 2) are put on binary
    grids on which every product and every partial sum of z -- 144 terms in a convolution layer, 4096 in a fully
    connected one -- is exact in float32 in any order."""
    wl = I.mixed(2)
    _announce(wl.name + " adjoint + gradient")
    data = dict(I.generate(wl))
    for k in ("W", "Wfc"):
        data[k] = (np.clip(np.round(data[k] * 128.0), -63, 63) / 128.0).astype(np.float32)
    for k in ("b", "bfc"):
        data[k] = (np.round(data[k] * 4096.0) / 4096.0).astype(np.float32)
    Ws, bs, kinds = I.per_layer_lists(wl, data)
    Uo, _, _ = _oracle_forward(wl, data)
    U = (np.clip(np.round(Uo * 32.0), -63, 63) / 32.0).astype(np.float32)
    del Uo
    lamN = (np.random.default_rng(21).standard_normal(wl.state_shape) / wl.B).astype(np.float32)
    gp = GpuMixed(wl, data)
    Lam, dW, db, dWfc, dbfc, hist, it = gp.adjoint(U, lamN)
    Lo, dWo, dbo, hist_o, _ = O.fas_adjoint(Ws, bs, U, lamN, wl.h, wl.m, wl.max_levels, wl.min_coarse, wl.relax,
                                            wl.max_iter, kinds, wl.act)
    eL = rel_l2_per_state(Lam, Lo)
    P = wl.fc_period
    conv = [n for n in range(wl.N) if n % P]
    eW = rel_l2_per_state(dW[conv], np.stack([dWo[n] for n in conv]))
    eb = rel_l2_per_state(db[conv], np.stack([dbo[n] for n in conv]))
    eWf = rel_l2_per_state(dWfc, np.stack([dWo[n] for n in range(0, wl.N, P)]))
    ebf = rel_l2_per_state(dbfc, np.stack([dbo[n] for n in range(0, wl.N, P)]))
    print(f"mixed adjoint: Lam {eL:.3e}  dW {eW:.3e}  db {eb:.3e}  dWfc {eWf:.3e}  dbfc {ebf:.3e}", flush=True)
    assert max(eL, eW, eb, eWf, ebf) <= 1e-5
    assert not dW[::P].any() and not db[::P].any()


def test_mixed_full_size_bf16_forward_and_adjoint_elementwise():
    """The same stack with bf16 operands (weights stored in bf16, states float): element by element at the bf16
    tolerance; the states to linearise about are bf16-representable so that both sides take every ReLU' decision
    on the same operand."""
    wl = I.mixed(2, I.BF16)
    _announce(wl.name)
    data = I.generate(wl)
    Ws, bs, kinds = I.per_layer_lists(wl, data)
    gp = GpuMixed(wl, data)
    U, hist, it = gp.forward()
    Uo, hist_o, _ = _oracle_forward(wl, data)
    err = rel_l2_per_state(U, Uo)
    inc = rel_l2_per_state(U[1:] - U[:-1], Uo[1:] - Uo[:-1])
    print(f"mixed bf16 forward: states {err:.3e}  increments {inc:.3e}", flush=True)
    assert err <= 2e-2 and it == 2
    for a, b in zip(hist, hist_o):
        assert abs(a - b) <= 5e-2 * b
    Ul = I.round_to_bf16(Uo.astype(np.float32))
    del Uo, U
    lamN = (np.random.default_rng(21).standard_normal(wl.state_shape) / wl.B).astype(np.float32)
    Lam, dW, db, dWfc, dbfc, _, _ = gp.adjoint(Ul, lamN)
    Lo, dWo, dbo, _, _ = O.fas_adjoint(Ws, bs, Ul, lamN, wl.h, wl.m, wl.max_levels, wl.min_coarse, wl.relax,
                                       wl.max_iter, kinds, wl.act)
    P = wl.fc_period
    conv = [n for n in range(wl.N) if n % P]
    errs = (rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW[conv], np.stack([dWo[n] for n in conv])),
            rel_l2_per_state(db[conv], np.stack([dbo[n] for n in conv])),
            rel_l2_per_state(dWfc, np.stack([dWo[n] for n in range(0, wl.N, P)])),
            rel_l2_per_state(dbfc, np.stack([dbo[n] for n in range(0, wl.N, P)])))
    print("mixed bf16 adjoint: Lam %.3e dW %.3e db %.3e dWfc %.3e dbfc %.3e" % errs, flush=True)
    assert max(errs) <= 2e-2
