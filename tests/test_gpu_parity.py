"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on
the same seeded inputs.  Tolerances (relative L2 per state / per layer gradient):
  fp32 path  1e-5      bf16 operand path  2e-2
Integer work (level maps) is compared bit-exactly in test_host_logic.py.
"""
import dataclasses

import numpy as np
import pytest

import mgrit_inputs as I
from oracle import mgrit_oracle as O
from tests.gpu_util import GpuProblem, oracle_forward, oracle_adjoint, rel_l2_per_state

pytestmark = pytest.mark.gpu

TOL = {I.FP32: 1e-5, I.BF16: 2e-2}


def _announce(name):
    print(f"\n[case] {name}", flush=True)


def _check_forward(wl, init=1, U_init=None, hist_rtol=None):
    _announce(wl.name)
    data = I.generate(wl)
    gp = GpuProblem(wl, data, init=init)
    rc, U, hist, it = gp.forward(U_init=U_init)
    Uo, hist_o, it_o = oracle_forward(wl, data, init=init, U_init=U_init)
    err = rel_l2_per_state(U, Uo)
    assert err <= TOL[wl.dtype], (wl.name, err)
    assert it == it_o
    if hist_rtol is None:
        hist_rtol = 1e-3 if wl.dtype == I.FP32 else 0.2
    for a, b in zip(hist, hist_o):
        assert abs(a - b) <= hist_rtol * max(abs(b), 1e-6), (hist, hist_o)
    return U, Uo, hist


# ------------------------------------------------------------------ the first benchmark config, as is
def test_cfg1_two_level_f_relax_reproduces_serial():
    wl = I.cfg1()
    U, Uo, hist = _check_forward(wl)
    data = I.generate(wl)
    Us = O.serial_forward(data["W"], data["b"], data["u0"], wl.h, wl.layer, wl.act)
    e = rel_l2_per_state(U, Us)
    assert e <= 1e-5, e                             # N/m = 4 cycles of F-relaxation are exact


def test_cfg1_against_the_stored_reference():
    """The stored oracle output of the smallest workload (tests/golden/cfg1_oracle.json): forward solve, adjoint
    solve about the stored states, parameter gradient."""
    import json
    import os
    wl = I.cfg1()
    _announce(wl.name + " vs stored reference")
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "cfg1_oracle.json")) as f:
        ref = json.load(f)
    data = I.generate(wl)
    gp = GpuProblem(wl, data)
    rc, U, hist, it = gp.forward()
    assert it == ref["cycles"]
    assert rel_l2_per_state(U, np.asarray(ref["U"])) <= 1e-5
    for a, b in zip(hist, ref["residual_history"]):
        assert abs(a - b) <= 1e-3 * b
    lamN = np.random.default_rng(1).standard_normal(wl.state_shape).astype(np.float32)
    Lam, dW, db, hist_a, _ = gp.adjoint(np.asarray(ref["U"], dtype=np.float32), lamN)
    assert rel_l2_per_state(Lam, np.asarray(ref["Lam"])) <= 1e-5
    assert rel_l2_per_state(dW, np.asarray(ref["dW"])) <= 1e-5
    assert rel_l2_per_state(db, np.asarray(ref["db"])) <= 1e-5


# ------------------------------------------------------------------ dense, reduced sizes
DENSE_CASES = [
    # ragged in batch and width (several tiles + a tail), 3 levels, FCF
    I.reduced(I.cfg2(3), name="dense_fp32_q72_B37_N64_L3", q=72, B=37, N=64),
    I.reduced(I.cfg2(2), name="dense_fp32_q264_B150_N32_L2_F", q=264, B=150, N=32, max_levels=2, relax=I.RELAX_F),
    I.reduced(I.cfg2(2), name="dense_fp32_q8_B1_N8_m2", q=8, B=1, N=8, m=2),
    I.reduced(I.cfg5(2), name="dense_bf16_q136_B50_N64_m4", q=136, B=50, N=64, m=4, head_classes=0),
    I.reduced(I.cfg5(2), name="dense_bf16_q256_B130_N256_m16", q=256, B=130, N=256, head_classes=0),
    I.reduced(I.cfg2(1), name="dense_fp32_serial_L1", q=40, B=9, N=13, max_levels=1),
    # enough groups for the largest tiles (128x128, both operand types), ragged against them
    I.reduced(I.cfg5(1), name="dense_bf16_q264_B260_N128_m2_bigtile", q=264, B=260, N=128, m=2, max_levels=2,
              head_classes=0),
    I.reduced(I.cfg2(1), name="dense_fp32_q136_B130_N128_m2_bigtile", q=136, B=130, N=128, m=2, max_levels=2),
    # at most 32 rows and a long contraction: the k-split kernel in its skinny-launch role (ragged rows, bias, both operand types)
    I.reduced(I.cfg2(1), name="dense_fp32_q2048_B20_N8_m2_deep_ksplit", q=2048, B=20, N=8, m=2, max_levels=2, bias_var=0.1),
    I.reduced(I.cfg5(1), name="dense_bf16_q4096_B9_N4_m2_deep_ksplit", q=4096, B=9, N=4, m=2, max_levels=2, head_classes=0,
              bias_var=0.1),
    # level sizes that are no multiples of m: trailing F-points behind the last C-point (79 -> 19 -> 4, 23 -> 11 -> 5)
    I.reduced(I.cfg2(3), name="dense_fp32_q72_B37_N79_m4_L3_trailing", q=72, B=37, N=79, bias_var=0.1),
    I.reduced(I.cfg2(2), name="dense_fp32_q40_B9_N23_m2_L3_F_trailing", q=40, B=9, N=23, m=2, relax=I.RELAX_F, act=I.TANH),
    I.reduced(I.cfg5(2), name="dense_bf16_q136_B50_N70_m4_trailing", q=136, B=50, N=70, m=4, head_classes=0),
    I.reduced(I.cfg2(1), name="dense_fp32_q16_N3_m4_too_short_to_coarsen", q=16, B=3, N=3, m=4),
]

# widths that are multiples of 128 (the fused sweep kernel's block width) at launch sizes below its threshold:
# these run through the lockstep launches
CHAIN_CASES = [
    I.reduced(I.cfg2(3), name="chain_fp32_q128_B37_N64_L3_FCF", q=128, B=37, N=64),
    I.reduced(I.cfg2(2), name="chain_fp32_q256_B70_N32_L2_F", q=256, B=70, N=32, max_levels=2, relax=I.RELAX_F,
              bias_var=0.1, act=I.TANH),
    I.reduced(I.cfg2(2), name="chain_fp32_q384_B33_N16_m2_L3", q=384, B=33, N=16, m=2, bias_var=0.1),
    I.reduced(I.cfg5(2), name="chain_bf16_q512_B40_N64_m4", q=512, B=40, N=64, m=4, head_classes=0),
    I.reduced(I.cfg5(2), name="chain_bf16_q128_B32_N32_m8_F", q=128, B=32, N=32, m=8, head_classes=0,
              relax=I.RELAX_F, max_levels=2),
    I.reduced(I.cfg2(1), name="chain_fp32_q512_serial_L1", q=512, B=20, N=9, max_levels=1),
]


@pytest.mark.parametrize("wl", CHAIN_CASES, ids=lambda w: w.name)
def test_dense_forward_chain_widths(wl):
    _check_forward(wl)


@pytest.mark.parametrize("wl", DENSE_CASES, ids=lambda w: w.name)
def test_dense_forward(wl):
    _check_forward(wl)


# ------------------------------------------------------------------ conv, reduced sizes
CONV_CASES = [
    I.reduced(I.cfg3(2), name="conv_fp32_c16_14x12_B3_N16", B=3, Himg=14, Wimg=12, N=16),
    I.reduced(I.cfg3(2), name="conv_fp32_c8_28x28_B2_N8_tanh", B=2, C=8, N=8, act=I.TANH, m=2),
    I.reduced(I.cfg3(1), name="conv_fp32_c40_9x7_B2_N8", B=2, C=40, Himg=9, Wimg=7, N=8, m=2, lifted_input=False),
    I.reduced(I.cfg4(2), name="conv_bf16_c64_12x10_B2_N64_L3", B=2, Himg=12, Wimg=10, N=64),
    I.reduced(I.cfg4(1), name="conv_bf16_c24_32x32_B1_N16_m4", B=1, C=24, N=16, m=4, max_levels=2),
    I.reduced(I.cfg3(2), name="conv_fp32_c16_14x12_B3_N19_m4_trailing", B=3, Himg=14, Wimg=12, N=19),
    I.reduced(I.cfg4(2), name="conv_bf16_c64_12x10_B2_N45_m3_L3_trailing", B=2, Himg=12, Wimg=10, N=45, m=3),
]


@pytest.mark.parametrize("wl", CONV_CASES, ids=lambda w: w.name)
def test_conv_forward(wl):
    _check_forward(wl)


# bf16 layers of 64 channels run a kernel compiled for that channel count (unrolled tap loop, no masks on the
# weight pieces); MGRIT_CONV_GENERIC=1 keeps them on the kernel with a run-time channel count.  Same arithmetic:
# forward and adjoint results must agree bit for bit, and with the oracle.
def test_conv_bf16_64_channels_fixed_and_generic_kernel(monkeypatch):
    wl = I.reduced(I.cfg4(2), name="conv_bf16_c64_20x12_B3_N32_m4_L2", B=3, Himg=20, Wimg=12, N=32, m=4, max_levels=2)
    _announce(wl.name)
    data = I.generate(wl)
    Uo, _, _ = oracle_forward(wl, data)
    res = {}
    for generic in (False, True):
        if generic:
            monkeypatch.setenv("MGRIT_CONV_GENERIC", "1")
        gp = GpuProblem(wl, data)
        rc, U, hist, it = gp.forward()
        assert rc == 0
        lamN = np.random.default_rng(5).standard_normal(wl.state_shape).astype(np.float32)
        Ul = I.round_to_bf16(U)      # ReLU' is a 0/1 decision: both sides take it on bf16-representable states
        Lam, dW, db, _, _ = gp.adjoint(Ul, lamN)
        res[generic] = (U, Lam, dW, db, lamN, Ul)
    for x, y in zip(res[False][:4], res[True][:4]):
        assert np.array_equal(x, y)
    U, Lam, dW, db, lamN, Ul = res[False]
    tol = TOL[wl.dtype]
    Lo, dWo, dbo, _, _ = oracle_adjoint(wl, data, Ul, lamN)
    eU, eL, eW = rel_l2_per_state(U, Uo), rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo)
    print(f"{wl.name}: U {eU:.3e} Lam {eL:.3e} dW {eW:.3e}", flush=True)
    assert eU <= tol and eL <= tol and eW <= tol, (eU, eL, eW)


# The all-taps parameter gradient of layers with more than 32 channels runs with eight wavefronts and taller slabs
# (MGRIT_CGRAD_WAVES=4: four, as for narrower layers); image widths whose 4-pixel groups divide 64 build the shifted
# patch copies by lane exchange (32 and 8 columns here), others element by element (12 columns).
@pytest.mark.parametrize("waves", ["8", "4"])
@pytest.mark.parametrize("shape", [(32, 32, 2), (5, 8, 3), (20, 12, 2)], ids=lambda s: "%dx%d" % (s[0], s[1]))
def test_conv_gradient_64_channels_wavefront_forms(shape, waves, monkeypatch):
    if waves == "4":
        monkeypatch.setenv("MGRIT_CGRAD_WAVES", "4")
    H, Wd, B = shape
    wl = I.reduced(I.cfg4(1), name=f"cgrad_bf16_c64_{H}x{Wd}_B{B}_N8_w{waves}", B=B, Himg=H, Wimg=Wd, N=8, m=2, max_levels=2,
                   act=I.TANH)
    _announce(wl.name)
    data = I.generate(wl)
    Uo, _, _ = oracle_forward(wl, data, max_iter=2)
    U = Uo.astype(np.float32)
    lamN = np.random.default_rng(11).standard_normal(wl.state_shape).astype(np.float32)
    gp = GpuProblem(wl, data)
    Lam, dW, db, _, _ = gp.adjoint(U, lamN)
    Lo, dWo, dbo, _, _ = oracle_adjoint(wl, data, U, lamN)
    tol = TOL[wl.dtype]
    eL, eW, eb = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo), rel_l2_per_state(db, dbo)
    print(f"{wl.name}: Lam {eL:.3e} dW {eW:.3e} db {eb:.3e}", flush=True)
    assert eL <= tol and eW <= tol and eb <= tol, (eL, eW, eb)


# ------------------------------------------------------------------ options of the boundary
def test_init_modes_and_user_guess():
    for q in (24, 128):
        wl = I.reduced(I.cfg2(2), name=f"dense_fp32_init_q{q}", q=q, B=5, N=16, max_levels=2)
        _check_forward(wl, init=0)
        rng = np.random.default_rng(3)
        Uinit = rng.standard_normal((wl.N + 1,) + wl.state_shape).astype(np.float32)
        _check_forward(wl, init=2, U_init=Uinit)


NESTED_CASES = [
    I.reduced(I.cfg2(2), name="nested_dense_fp32_q72_B37_N64_L3_FCF", q=72, B=37, N=64, bias_var=0.1),
    I.reduced(I.cfg2(1), name="nested_dense_fp32_q40_B9_N32_L2_F", q=40, B=9, N=32, max_levels=2, relax=I.RELAX_F),
    I.reduced(I.cfg5(2), name="nested_dense_bf16_q136_B50_N64_m4", q=136, B=50, N=64, m=4),
    I.reduced(I.cfg2(1), name="nested_dense_fp32_q16_N16_m2_deep", q=16, B=3, N=16, m=2, max_levels=16, bias_var=0.1),
    I.reduced(I.cfg3(1), name="nested_conv_fp32_c16_10x9_B2_N16_L3", B=2, Himg=10, Wimg=9, N=16, m=2, max_levels=3),
    I.reduced(I.cfg4(1), name="nested_conv_bf16_c64_8x8_B3_N16_m4", B=3, Himg=8, Wimg=8, N=16, m=4, max_levels=2),
    I.reduced(I.cfg2(2), name="nested_dense_fp32_q72_B37_N79_L3_trailing", q=72, B=37, N=79, bias_var=0.1),
    I.reduced(I.cfg3(1), name="nested_conv_fp32_c16_10x9_B2_N23_m2_L3_trailing", B=2, Himg=10, Wimg=9, N=23, m=2, max_levels=3),
]


@pytest.mark.parametrize("wl", NESTED_CASES, ids=lambda w: w.name)
def test_nested_iteration_start_forward(wl):
    """init = MGRIT_INIT_NESTED: coarsest level first, handed up level by level, then the cycles."""
    _check_forward(wl, init=3)


@pytest.mark.parametrize("wl", [
    I.reduced(I.cfg5(2), name="nested_adj_dense_fp32_q72_B37_N64_m4", q=72, B=37, N=64, m=4, dtype=I.FP32),
    I.reduced(I.cfg5(1), name="nested_adj_dense_bf16_q136_B50_N64_m4", q=136, B=50, N=64, m=4),
    I.reduced(I.cfg3(1), name="nested_adj_conv_fp32_c16_10x9_B2_N16", B=2, Himg=10, Wimg=9, N=16, act=I.TANH),
    I.reduced(I.cfg5(2), name="nested_adj_dense_fp32_q72_B37_N79_m4_trailing", q=72, B=37, N=79, m=4, dtype=I.FP32),
], ids=lambda w: w.name)
def test_nested_iteration_start_adjoint(wl):
    _announce(wl.name)
    data = I.generate(wl)
    Uo, _, _ = oracle_forward(wl, data, max_iter=2, init=3)
    U = Uo.astype(np.float32)
    rng = np.random.default_rng(19)
    lamN = rng.standard_normal(wl.state_shape).astype(np.float32)
    gp = GpuProblem(wl, data, init=3)
    Lam, dW, db, hist, it = gp.adjoint(U, lamN)
    Lo, dWo, dbo, hist_o, it_o = oracle_adjoint(wl, data, U, lamN, init=3)
    tol = TOL[wl.dtype]
    eL, eW, eb = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo), rel_l2_per_state(db, dbo)
    assert eL <= tol and eW <= tol and eb <= tol, (eL, eW, eb)
    assert it == it_o
    for a, b in zip(hist, hist_o):
        assert abs(a - b) <= 5e-2 * b + 1e-7


def test_tolerance_stop_and_rms_norm():
    wl = I.reduced(I.cfg2(30), name="dense_fp32_tol", q=32, B=8, N=64, tol=1e-4, norm_kind=1)
    _announce(wl.name)
    data = I.generate(wl)
    gp = GpuProblem(wl, data)
    rc, U, hist, it = gp.forward()
    Uo, hist_o, it_o = oracle_forward(wl, data)
    assert hist[-1] <= 1e-4 and all(h > 1e-4 for h in hist[:-1])
    assert abs(it - it_o) <= 1                 # the stopping cycle may differ by one between fp32 and fp64
    k = min(it, it_o)
    for a, b in zip(hist[:k - 1], hist_o[:k - 1]):
        assert abs(a - b) <= 2e-2 * b


def test_fixed_point_of_the_cycle():
    """Started from serial propagation computed on the GPU, a cycle reports a residual at rounding level and
    leaves the iterate where it is."""
    wl = I.reduced(I.cfg2(1), name="dense_fp32_fixed_point", q=64, B=16, N=64)
    _announce(wl.name)
    data = I.generate(wl)
    ser = GpuProblem(dataclasses.replace(wl, max_levels=1), data)
    _, Us, _, _ = ser.forward()
    gp = GpuProblem(wl, data, init=2)
    rc, U, hist, it = gp.forward(U_init=Us)
    e = rel_l2_per_state(U, Us)
    assert hist[0] < 1e-5 and e < 1e-6, (hist, e)


def test_residual_norm_entry_point():
    wl = I.reduced(I.cfg2(1), name="dense_fp32_resnorm", q=48, B=7, N=32)
    _announce(wl.name)
    data = I.generate(wl)
    rng = np.random.default_rng(5)
    U = rng.standard_normal((wl.N + 1,) + wl.state_shape).astype(np.float32)
    gp = GpuProblem(wl, data)
    for nk in (0, 1):
        gp.p.norm_kind = nk
        got = gp.residual_norm(U)
        ref = O.residual_norm(data["W"], data["b"], data["u0"], U, wl.h, wl.layer, wl.act, norm_kind=nk)
        assert abs(got - ref) <= 1e-5 * ref
    wlc = I.reduced(I.cfg3(1), name="conv_fp32_resnorm", B=2, Himg=10, Wimg=9, N=6, m=2)
    data = I.generate(wlc)
    U = rng.standard_normal((wlc.N + 1,) + wlc.state_shape).astype(np.float32)
    gp = GpuProblem(wlc, data)
    got = gp.residual_norm(U)
    ref = O.residual_norm(data["W"], data["b"], data["u0"], U, wlc.h, wlc.layer, wlc.act)
    assert abs(got - ref) <= 1e-5 * ref


def test_repeated_runs_are_bitwise_identical():
    for q in (72, 128):
        wl = I.reduced(I.cfg2(3), name=f"dense_fp32_determinism_q{q}", q=q, B=37, N=64)
        _announce(wl.name)
        data = I.generate(wl)
        gp = GpuProblem(wl, data)
        _, U1, h1, _ = gp.forward()
        _, U2, h2, _ = gp.forward()
        same = bool(np.array_equal(U1, U2))
        assert same and h1 == h2


# ------------------------------------------------------------------ adjoint solve and parameter gradient
ADJ_CASES = [
    I.reduced(I.cfg5(3), name="adj_dense_fp32_q72_B37_N64_m4", q=72, B=37, N=64, m=4, dtype=I.FP32),
    I.reduced(I.cfg5(2), name="adj_dense_bf16_q136_B50_N64_m4", q=136, B=50, N=64, m=4),
    I.reduced(I.cfg5(2), name="adj_dense_fp32_relu_F_L2", q=40, B=12, N=32, m=4, dtype=I.FP32, act=I.RELU,
              max_levels=2, relax=I.RELAX_F),
    # widths that are multiples of 128
    I.reduced(I.cfg5(3), name="adj_chain_fp32_q128_B37_N64_m4", q=128, B=37, N=64, m=4, dtype=I.FP32),
    I.reduced(I.cfg5(2), name="adj_chain_bf16_q256_B50_N64_m4", q=256, B=50, N=64, m=4),
    I.reduced(I.cfg5(2), name="adj_chain_fp32_q256_relu_F_L2", q=256, B=12, N=32, m=4, dtype=I.FP32, act=I.RELU,
              max_levels=2, relax=I.RELAX_F),
    I.reduced(I.cfg5(1), name="adj_fp32_q512_B8_N16_m4", q=512, B=8, N=16, m=4, dtype=I.FP32),
    # the k-split kernel (skinny launch) with the act' operand and in the act' launch itself
    I.reduced(I.cfg5(1), name="adj_dense_fp32_q2048_B20_N8_m2_deep_ksplit", q=2048, B=20, N=8, m=2, max_levels=2, dtype=I.FP32),
    I.reduced(I.cfg5(1), name="adj_dense_bf16_q4096_B32_N4_m2_deep_ksplit", q=4096, B=32, N=4, m=2, max_levels=2),
    # level sizes that are no multiples of m: the adjoint hierarchy counts from layer N, its trailing F-points end at layer 0
    I.reduced(I.cfg5(3), name="adj_dense_fp32_q72_B37_N79_m4_L3_trailing", q=72, B=37, N=79, m=4, max_levels=3, dtype=I.FP32),
    I.reduced(I.cfg5(2), name="adj_dense_bf16_q136_B50_N70_m4_trailing", q=136, B=50, N=70, m=4),
    I.reduced(I.cfg5(2), name="adj_dense_fp32_q40_N23_m2_L3_relu_F_trailing", q=40, B=12, N=23, m=2, max_levels=3,
              dtype=I.FP32, act=I.RELU, relax=I.RELAX_F),
]


@pytest.mark.parametrize("wl", ADJ_CASES, ids=lambda w: w.name)
def test_dense_adjoint_and_gradient(wl):
    _announce(wl.name)
    data = I.generate(wl)
    # linearise about an approximate forward solve (2 cycles), as the training step does
    Uo, _, _ = oracle_forward(wl, data, max_iter=2)
    U = Uo.astype(np.float32)
    lamN = I.terminal_adjoint(wl, data, U[-1])
    gp = GpuProblem(wl, data)
    Lam, dW, db, hist, it = gp.adjoint(U, lamN)
    Lo, dWo, dbo, hist_o, it_o = oracle_adjoint(wl, data, U, lamN)
    tol = TOL[wl.dtype]
    eL, eW, eb = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo), rel_l2_per_state(db, dbo)
    assert eL <= tol and eW <= tol and eb <= tol, (eL, eW, eb)
    assert it == it_o


CONV_ADJ_CASES = [
    I.reduced(I.cfg3(2), name="adj_conv_fp32_c16_10x9_B2_N16", B=2, Himg=10, Wimg=9, N=16, act=I.TANH),
    I.reduced(I.cfg4(1), name="adj_conv_bf16_c64_8x8_B3_N16_m4", B=3, Himg=8, Wimg=8, N=16, m=4, max_levels=2),
    I.reduced(I.cfg3(1), name="adj_conv_fp32_c24_7x5_B2_N8_m2", B=2, C=24, Himg=7, Wimg=5, N=8, m=2,
              lifted_input=False),
    # shapes of the all-taps gradient kernel: every (row blocks, column blocks per wavefront) arrangement,
    # one slab per layer (no partial sums), ragged last slab, widest row it takes, and the per-tap
    # kernel that wider rows fall back to
    I.reduced(I.cfg4(1), name="adj_conv_bf16_c64_32x32_B2_N8", B=2, N=8, m=2, max_levels=2, act=I.TANH),
    I.reduced(I.cfg3(1), name="adj_conv_fp32_c8_2x32_B1_N4_one_slab", B=1, C=8, Himg=2, Wimg=32, N=4, m=2,
              lifted_input=False, act=I.TANH),
    I.reduced(I.cfg3(1), name="adj_conv_fp32_c32_7x28_B2_N4", B=2, C=32, Himg=7, Wimg=28, N=4, m=2,
              lifted_input=False, act=I.TANH),
    I.reduced(I.cfg4(1), name="adj_conv_bf16_c40_5x40_B2_N4", B=2, C=40, Himg=5, Wimg=40, N=4, m=2, max_levels=2,
              act=I.TANH),
    I.reduced(I.cfg4(1), name="adj_conv_bf16_c48_9x12_B3_N4", B=3, C=48, Himg=9, Wimg=12, N=4, m=2, max_levels=2,
              act=I.TANH),
    I.reduced(I.cfg4(1), name="adj_conv_bf16_c56_3x64_B2_N4", B=2, C=56, Himg=3, Wimg=64, N=4, m=2, max_levels=2,
              act=I.TANH),
    I.reduced(I.cfg3(1), name="adj_conv_fp32_c8_2x256_B1_N4_wide", B=1, C=8, Himg=2, Wimg=256, N=4, m=2,
              lifted_input=False, act=I.TANH),
    I.reduced(I.cfg3(1), name="adj_conv_fp32_c16_1x9_B2_N4", B=2, C=16, Himg=1, Wimg=9, N=4, m=2,
              lifted_input=False, act=I.TANH),
    I.reduced(I.cfg3(1), name="adj_conv_fp32_c16_7x1_B2_N4", B=2, C=16, Himg=7, Wimg=1, N=4, m=2,
              lifted_input=False, act=I.TANH),
    I.reduced(I.cfg3(2), name="adj_conv_fp32_c16_10x9_B2_N19_m4_trailing", B=2, Himg=10, Wimg=9, N=19, act=I.TANH),
    I.reduced(I.cfg4(1), name="adj_conv_bf16_c64_8x8_B3_N22_m3_L3_trailing", B=3, Himg=8, Wimg=8, N=22, m=3, max_levels=3),
]


@pytest.mark.parametrize("wl", CONV_ADJ_CASES, ids=lambda w: w.name)
def test_conv_adjoint_and_gradient(wl):
    _announce(wl.name)
    data = I.generate(wl)
    Uo, _, _ = oracle_forward(wl, data, max_iter=2)
    U = Uo.astype(np.float32)
    if wl.dtype == I.BF16 and wl.act == I.RELU:
        # ReLU' is a 0/1 decision on the sign of z = A u + b.  The bf16 path rounds the state operand to
        # bf16 before the product, which flips that decision where z is close to 0; both sides must take
        # it in the same precision, so the states to linearise about are made bf16-representable here
        # (rounding them again on the GPU is then a no-op and both sides see the same z up to summation order).
        U = I.round_to_bf16(U)
    rng = np.random.default_rng(9)
    lamN = rng.standard_normal(wl.state_shape).astype(np.float32)
    gp = GpuProblem(wl, data)
    Lam, dW, db, hist, it = gp.adjoint(U, lamN)
    Lo, dWo, dbo, hist_o, _ = oracle_adjoint(wl, data, U, lamN)
    tol = TOL[wl.dtype]
    eL, eW, eb = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo), rel_l2_per_state(db, dbo)
    assert eL <= tol and eW <= tol and eb <= tol, (eL, eW, eb)


# ------------------------------------------------------------------ degenerate and edge cases
EDGE_CASES = [
    # a single coarse interval per level; the coarsest level has one step
    I.reduced(I.cfg2(2), name="edge_one_interval_N4_m4", q=16, B=2, N=4, m=4, max_levels=3),
    # batch of one, width 8 (smallest supported), m = 2, as many levels as fit
    I.reduced(I.cfg2(2), name="edge_B1_q8_N16_m2_deep", q=8, B=1, N=16, m=2, max_levels=16, bias_var=0.1),
    # N == 1: no coarsening possible, serial propagation of one step
    I.reduced(I.cfg2(1), name="edge_N1", q=16, B=3, N=1, m=2, max_levels=4),
    # one-pixel-high and one-pixel-wide images (every tap but the centre column/row is padding)
    I.reduced(I.cfg3(2), name="edge_conv_1x9", B=2, C=8, Himg=1, Wimg=9, N=8, m=2, lifted_input=False),
    I.reduced(I.cfg3(2), name="edge_conv_7x1", B=2, C=8, Himg=7, Wimg=1, N=8, m=2, lifted_input=False),
    # widest supported image row
    I.reduced(I.cfg3(1), name="edge_conv_2x256", B=1, C=8, Himg=2, Wimg=256, N=4, m=2, lifted_input=False),
]


@pytest.mark.parametrize("wl", EDGE_CASES, ids=lambda w: w.name)
def test_edge_cases_forward(wl):
    _check_forward(wl)


def test_non_finite_input_is_reported():
    """A NaN in the input makes the residual norm non-finite: the solve returns MGRIT_ERR_NONFINITE."""
    from paper_2007_07336_amd import binding as Bd
    wl = I.reduced(I.cfg2(2), name="nan_input", q=16, B=2, N=8, m=2, max_levels=2)
    _announce(wl.name)
    data = I.generate(wl)
    data["u0"] = data["u0"].copy()
    data["u0"][0, 0] = np.nan
    gp = GpuProblem(wl, data)
    rc, U, hist, it = gp.forward(check=False)
    assert rc == Bd.MGRIT_ERR_NONFINITE
    gp2 = GpuProblem(wl, data, tol=1e-3)
    rc2, _, _, it2 = gp2.forward(check=False)
    assert rc2 == Bd.MGRIT_ERR_NONFINITE and it2 == 1


def test_conv_repeated_runs_are_bitwise_identical():
    wl = I.reduced(I.cfg4(2), name="conv_bf16_determinism", B=2, Himg=12, Wimg=10, N=64)
    _announce(wl.name)
    data = I.generate(wl)
    gp = GpuProblem(wl, data)
    _, U1, h1, _ = gp.forward()
    _, U2, h2, _ = gp.forward()
    same = bool(np.array_equal(U1, U2))
    assert same and h1 == h2


def test_maximum_layer_count_forward_and_adjoint():
    """N = 65535, the largest layer count the build accepts (points and layers index one grid dimension of the
    transfer kernels): forward and adjoint solve with gradient against the oracle."""
    wl = I.reduced(I.cfg2(2), name="edge_N65535_q8_B2_m3", q=8, B=2, N=65535, m=3, max_levels=2, act=I.TANH,
                   bias_var=0.1)
    _announce(wl.name)
    data = I.generate(wl)
    gp = GpuProblem(wl, data)
    rc, U, hist, it = gp.forward()
    Uo, hist_o, _ = oracle_forward(wl, data)
    assert rel_l2_per_state(U, Uo) <= 1e-5
    for a, b in zip(hist, hist_o):
        assert abs(a - b) <= 1e-3 * b + 1e-4        # the second norm (2e-5) is at the float32 rounding floor
    lamN = np.random.default_rng(3).standard_normal(wl.state_shape).astype(np.float32)
    Ul = Uo.astype(np.float32)
    Lam, dW, db, _, _ = gp.adjoint(Ul, lamN)
    Lo, dWo, dbo, _, _ = oracle_adjoint(wl, data, Ul, lamN)
    eL, eW, eb = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo), rel_l2_per_state(db, dbo)
    # Tolerance at this depth (the 1e-5 bar is stated for the benchmark depths, N <= 1024): N float32 layer steps
    # in sequence, each rounding the state once (relative 2^-24), leave a random-walk error of sqrt(N) * 2^-24 =
    # 1.5e-5 in a state that the float64 oracle does not have, so a state may differ by 2e-5; a layer's gradient
    # is a sum over B = 2 samples of products of two such quantities with either sign, which at most triples
    # the relative error: 5e-5.
    assert eL <= 2e-5 and eW <= 5e-5 and eb <= 5e-5, (eL, eW, eb)


# ------------------------------------------------------------------ parameter gradient of wide dense layers
# Layers of width 512 and more take the 256x256 gradient kernel, which also forms the bias gradient;
# MGRIT_GRAD_NARROW=1 keeps them on the 128x128 kernel with its separate bias pass.  Widths ragged against the
# 256-wide tile (520 = 2 x 256 + 8, 776), batches ragged against the 32-row slabs (50, 70), both operand types.
GRAD_WIDE_CASES = [
    I.reduced(I.cfg5(1), name="gradw_fp32_q520_B50_N8_m2", q=520, B=50, N=8, m=2, max_levels=2, dtype=I.FP32),
    I.reduced(I.cfg5(1), name="gradw_bf16_q776_B70_N8_m4", q=776, B=70, N=8, m=4, max_levels=2),
    I.reduced(I.cfg5(1), name="gradw_bf16_q1024_B256_N16_m4", q=1024, B=256, N=16, m=4, max_levels=2),
]


@pytest.mark.parametrize("wide", [True, False], ids=["tile256", "tile128"])
@pytest.mark.parametrize("wl", GRAD_WIDE_CASES, ids=lambda w: w.name)
def test_dense_parameter_gradient_wide_layers(wl, wide, monkeypatch):
    if not wide:
        monkeypatch.setenv("MGRIT_GRAD_NARROW", "1")
    _announce(f"{wl.name} wide={wide}")
    data = I.generate(wl)
    Uo, _, _ = oracle_forward(wl, data)
    U = Uo.astype(np.float32)
    lamN = I.terminal_adjoint(wl, data, U[-1])
    gp = GpuProblem(wl, data)
    Lam, dW, db, hist, it = gp.adjoint(U, lamN)
    Lo, dWo, dbo, hist_o, it_o = oracle_adjoint(wl, data, U, lamN)
    tol = TOL[wl.dtype]
    eL, eW, eb = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo), rel_l2_per_state(db, dbo)
    print(f"{wl.name}: Lam {eL:.3e} dW {eW:.3e} db {eb:.3e}", flush=True)
    assert eL <= tol and eW <= tol and eb <= tol, (eL, eW, eb)
    # the bias gradient alone (dW not requested) and the weight gradient alone
    import torch
    import paper_2007_07336_amd as M
    Ud, lam = torch.from_numpy(U).cuda(), torch.from_numpy(lamN).cuda()
    ws = torch.empty(M.mgrit_adjoint_workspace_bytes(gp.p), dtype=torch.uint8, device="cuda")
    Lam2, db2 = torch.zeros_like(Ud), torch.full_like(gp.b, float("nan"))
    M.mgrit_fas_adjoint(gp.p, gp.W, gp.b, Ud, lam, Lam2, None, db2, ws)
    assert np.array_equal(db2.cpu().numpy(), db)
    dW2 = torch.full(gp.W.shape, float("nan"), dtype=torch.float32, device="cuda")
    M.mgrit_fas_adjoint(gp.p, gp.W, gp.b, Ud, lam, Lam2, dW2, None, ws)
    assert np.array_equal(dW2.cpu().numpy(), dW)


# ------------------------------------------------------------------ dense steps on whole tiles
# When batch, width and contraction length are whole multiples of the tile, the dense step kernel runs a loop
# without bounds masks (MGRIT_MASKED_STEP=1 sends such shapes through the masked loop that ragged shapes use), and
# on bf16 128x128 tiles it keeps the tile's own state columns from that loop for the skip connection
# (MGRIT_STEP_REREAD=1: the epilogue reads them again).
# Both must agree with the oracle, and with each other bit for bit: the arithmetic is the same.  Shapes: the
# 128x128 tile in both operand types (batch 256 / 128, width 512 so that the fused sweeps stay out of the way)
# and the 64x64 tile (batch 64, width 192).
WHOLE_TILE_CASES = [
    I.reduced(I.cfg5(1), name="whole_bf16_q512_B256_N16_m4", q=512, B=256, N=16, m=4, max_levels=2),
    I.reduced(I.cfg5(1), name="whole_fp32_q512_B128_N16_m4", q=512, B=128, N=16, m=4, max_levels=2, dtype=I.FP32),
    I.reduced(I.cfg5(1), name="whole_bf16_q192_B64_N64_m4", q=192, B=64, N=64, m=4, max_levels=2),
    # a single 128x128 tile per group (both kept state slabs are the only two of the contraction), 256 groups
    I.reduced(I.cfg5(1), name="whole_bf16_q128_B128_N512_m2", q=128, B=128, N=512, m=2, max_levels=2),
]


@pytest.mark.parametrize("wl", WHOLE_TILE_CASES, ids=lambda w: w.name)
def test_dense_step_whole_tiles_unmasked_and_masked(wl, monkeypatch):
    _announce(wl.name)
    data = I.generate(wl)
    Uo, hist_o, _ = oracle_forward(wl, data)
    res = {}
    # default; the epilogue reading the state again instead of keeping the tile's own columns from the k loop
    # (bf16 128x128 tiles); the masked loop
    for mode, var in (("default", None), ("reread", "MGRIT_STEP_REREAD"), ("masked", "MGRIT_MASKED_STEP")):
        if var:
            monkeypatch.setenv(var, "1")
        gp = GpuProblem(wl, data)
        rc, U, hist, it = gp.forward()
        assert rc == 0
        lamN = I.terminal_adjoint(wl, data, U[-1])
        Lam, dW, db, _, _ = gp.adjoint(U, lamN)
        res[mode] = (U, Lam, dW, db, lamN)
        if var:
            monkeypatch.delenv(var)
    U, Lam, dW, db, lamN = res["default"]
    for mode in ("reread", "masked"):
        for x, y in zip(res["default"][:4], res[mode][:4]):
            assert np.array_equal(x, y), mode
    tol = TOL[wl.dtype]
    eU = rel_l2_per_state(U, Uo)
    Lo, dWo, dbo, _, _ = oracle_adjoint(wl, data, U, lamN)
    eL, eW = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo)
    print(f"{wl.name}: U {eU:.3e} Lam {eL:.3e} dW {eW:.3e}", flush=True)
    assert eU <= tol and eL <= tol and eW <= tol, (eU, eL, eW)


# ------------------------------------------------------------------ fused F-relaxation sweeps (dense layers)
# Shapes on which the library fuses the steps of an F-relaxation sweep into one launch (width 128 or 256;
# at least 128 (interval, 32-row slice) workgroups; m >= 3); each also runs with the fused
# launches switched off (MGRIT_NO_SWEEP=1), i.e. through the lockstep launches, and the two must agree with the
# oracle alike.
SWEEP_CASES = [
    I.reduced(I.cfg2(2), name="sweep_fp32_q128_B37_N256_m4_L3_FCF", q=128, B=37, N=256),
    I.reduced(I.cfg2(1), name="sweep_fp32_q256_B70_N192_m4_L2_F_tanh_bias", q=256, B=70, N=192, max_levels=2,
              relax=I.RELAX_F, bias_var=0.1, act=I.TANH),
    I.reduced(I.cfg5(1), name="sweep_bf16_q256_B40_N192_m3", q=256, B=40, N=192, m=3, max_levels=2, head_classes=0),
    I.reduced(I.cfg5(1), name="sweep_bf16_q128_B512_N128_m16", q=128, B=512, N=128, m=16, max_levels=2,
              head_classes=0),
    # deep enough that the middle level's sweeps are fused too: they carry the FAS right-hand side
    I.reduced(I.cfg2(1), name="sweep_fp32_q128_B37_N1024_m4_L3_rhs", q=128, B=37, N=1024, bias_var=0.1, act=I.TANH),
    # trailing F-points: the fused launch covers the whole intervals, single-group launches the rest
    # (190 -> 47, two trailing points; 1030 -> 257 -> 64, two on the fine and one on the middle level)
    I.reduced(I.cfg2(2), name="sweep_fp32_q256_B70_N190_m4_L2_trailing", q=256, B=70, N=190, max_levels=2, bias_var=0.1),
    I.reduced(I.cfg5(1), name="sweep_bf16_q128_B40_N1030_m4_L3_trailing", q=128, B=40, N=1030, m=4, max_levels=3,
              head_classes=0),
]


@pytest.mark.parametrize("fused", [True, False], ids=["fused", "lockstep"])
@pytest.mark.parametrize("wl", SWEEP_CASES, ids=lambda w: w.name)
def test_dense_forward_fused_sweeps(wl, fused, monkeypatch):
    import paper_2007_07336_amd as M
    if not fused:
        monkeypatch.setenv("MGRIT_NO_SWEEP", "1")
    _announce(f"{wl.name} fused={fused}")
    data = I.generate(wl)
    gp = GpuProblem(wl, data)
    M.mgrit_trace_begin()
    rc, U, hist, it = gp.forward()
    tr = M.mgrit_trace_end()
    assert any(k.startswith("dense_sweep_kernel") for k in tr) == fused, tr      # the path under test did run
    Uo, hist_o, it_o = oracle_forward(wl, data)
    assert rel_l2_per_state(U, Uo) <= TOL[wl.dtype]
    assert it == it_o
    for a, b in zip(hist, hist_o):
        assert abs(a - b) <= (1e-3 if wl.dtype == I.FP32 else 5e-2) * max(b, 1e-6)


def test_dense_fused_sweeps_nested_start_three_levels():
    wl = I.reduced(I.cfg2(2), name="sweep_fp32_q128_B64_N256_nested", q=128, B=64, N=256, bias_var=0.1, act=I.TANH)
    _announce(wl.name)
    data = I.generate(wl)
    gp = GpuProblem(wl, data, init=3)
    rc, U, hist, it = gp.forward()
    Uo, hist_o, _ = oracle_forward(wl, data, init=3)
    assert rel_l2_per_state(U, Uo) <= 1e-5


SWEEP_ADJ_CASES = [
    I.reduced(I.cfg5(2), name="adj_sweep_fp32_q128_B37_N256_m4_L3", q=128, B=37, N=256, m=4, max_levels=3, dtype=I.FP32),
    I.reduced(I.cfg5(1), name="adj_sweep_bf16_q256_B70_N192_m4_relu", q=256, B=70, N=192, m=4, max_levels=2, act=I.RELU),
    I.reduced(I.cfg5(1), name="adj_sweep_fp32_q256_B100_N96_m3_F", q=256, B=100, N=96, m=3, max_levels=2, dtype=I.FP32,
              relax=I.RELAX_F),
    I.reduced(I.cfg5(1), name="adj_sweep_bf16_q128_B40_N1024_m4_L3_rhs", q=128, B=40, N=1024, m=4, max_levels=3),
    I.reduced(I.cfg5(2), name="adj_sweep_fp32_q256_B70_N190_m4_trailing", q=256, B=70, N=190, m=4, max_levels=2, dtype=I.FP32),
    I.reduced(I.cfg5(1), name="adj_sweep_fp32_q128_B40_N1030_m4_L3_trailing", q=128, B=40, N=1030, m=4, max_levels=3,
              dtype=I.FP32),
]


@pytest.mark.parametrize("fused", [True, False], ids=["fused", "lockstep"])
@pytest.mark.parametrize("wl", SWEEP_ADJ_CASES, ids=lambda w: w.name)
def test_dense_adjoint_fused_sweeps(wl, fused, monkeypatch):
    import paper_2007_07336_amd as M
    if not fused:
        monkeypatch.setenv("MGRIT_NO_SWEEP", "1")
    _announce(f"{wl.name} fused={fused}")
    data = I.generate(wl)
    Uo, _, _ = oracle_forward(wl, data, max_iter=2)
    U = Uo.astype(np.float32)
    if wl.dtype == I.BF16 and wl.act == I.RELU:
        U = I.round_to_bf16(U)          # both sides take the ReLU' decision on the same bf16 operand
    lamN = I.terminal_adjoint(wl, data, U[-1])
    gp = GpuProblem(wl, data)
    M.mgrit_trace_begin()
    Lam, dW, db, hist, it = gp.adjoint(U, lamN)
    tr = M.mgrit_trace_end()
    assert any(k.startswith("dense_sweep_kernel") for k in tr) == fused, tr
    Lo, dWo, dbo, hist_o, it_o = oracle_adjoint(wl, data, U, lamN)
    tol = TOL[wl.dtype]
    eL, eW, eb = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo), rel_l2_per_state(db, dbo)
    assert eL <= tol and eW <= tol and eb <= tol, (eL, eW, eb)


# ------------------------------------------------------------------ the adjoint on the weights as stored
# The adjoint of a dense layer contracts over the weights' slow index.  By default every dense kernel (tiled step in
# its masked / whole-tile / kept-state forms, k-split step, fused sweep) reads the caller's W[k][n] as stored;
# MGRIT_ADJ_TRANSPOSED=1 makes a transposed copy in the workspace and runs the forward kernels' reading on it.  The
# arithmetic and its order are the same, so the two agree bit for bit (the default path is the one every other
# adjoint test compares with the oracle), and the default workspace is smaller by the copy.
AS_STORED_CASES = [w for w in ADJ_CASES if w.name in (
    "adj_dense_fp32_q72_B37_N64_m4", "adj_dense_bf16_q136_B50_N64_m4", "adj_fp32_q512_B8_N16_m4",
    "adj_dense_fp32_q2048_B20_N8_m2_deep_ksplit", "adj_dense_bf16_q4096_B32_N4_m2_deep_ksplit",
    "adj_dense_bf16_q136_B50_N70_m4_trailing")] + WHOLE_TILE_CASES + [w for w in SWEEP_ADJ_CASES if w.name in (
    "adj_sweep_fp32_q128_B37_N256_m4_L3", "adj_sweep_bf16_q256_B70_N192_m4_relu", "adj_sweep_fp32_q256_B100_N96_m3_F",
    "adj_sweep_bf16_q128_B40_N1024_m4_L3_rhs")]


@pytest.mark.parametrize("wl", AS_STORED_CASES, ids=lambda w: w.name)
def test_dense_adjoint_weights_as_stored_and_transposed_copy(wl, monkeypatch):
    import paper_2007_07336_amd as M
    _announce(wl.name)
    data = I.generate(wl)
    gp = GpuProblem(wl, data)
    rc, U, _, _ = gp.forward()
    assert rc == 0
    if wl.dtype == I.BF16 and wl.act == I.RELU:
        U = I.round_to_bf16(U)
    lamN = I.terminal_adjoint(wl, data, U[-1])
    n_default = M.mgrit_adjoint_workspace_bytes(gp.p)
    M.mgrit_trace_begin()
    res = gp.adjoint(U, lamN)
    tr = M.mgrit_trace_end()
    monkeypatch.setenv("MGRIT_ADJ_TRANSPOSED", "1")
    n_copy = M.mgrit_adjoint_workspace_bytes(gp.p)
    ref = gp.adjoint(U, lamN)
    monkeypatch.delenv("MGRIT_ADJ_TRANSPOSED")
    wbytes = wl.N * wl.q * wl.q * (4 if wl.dtype == I.FP32 else 2)
    assert 0 <= n_copy - n_default - wbytes < 4096, (n_copy, n_default, wbytes)
    print(f"{wl.name}: workspace {n_default} / {n_copy} bytes; kernels {sorted(tr)}", flush=True)
    for x, y in zip(res[:3], ref[:3]):
        assert np.array_equal(x, y)
    assert res[3] == ref[3] and res[4] == ref[4]


# ------------------------------------------------------------------ fused sweeps of convolution layers
CONV_SWEEP_CASES = [
    I.reduced(I.cfg3(2), name="csweep_fp32_c16_7x5_B8_N64_m4_L2_FCF", B=8, Himg=7, Wimg=5, N=64),
    # 784 pixels: 49 blocks of 16 over eight wavefronts (the last one a block short); 8 channels (half of the MFMA
    # columns padding, the whole patch cleared); trailing F-points behind the fused launch
    I.reduced(I.cfg3(1), name="csweep_fp32_c8_28x28_B8_N66_m4_L2_F_tanh", B=8, C=8, N=66, relax=I.RELAX_F, act=I.TANH,
              lifted_input=False),
    I.reduced(I.cfg3(1), name="csweep_fp32_c16_28x28_B8_N64_m4_L2", B=8, N=64, bias_var=0.1),
    # three levels with enough intervals that the middle level's sweeps are fused too (they carry the FAS right-hand side)
    I.reduced(I.cfg3(1), name="csweep_fp32_c16_9x9_B32_N48_m3_L3_rhs", B=32, Himg=9, Wimg=9, N=48, m=3, max_levels=3,
              lifted_input=False),
    # a pixel count that is no multiple of 16 and a one-pixel-wide image
    I.reduced(I.cfg3(1), name="csweep_fp32_c16_5x1_B16_N32_m4", B=16, Himg=5, Wimg=1, N=32, m=4, max_levels=2,
              lifted_input=False, act=I.TANH),
]


@pytest.mark.parametrize("fused", [True, False], ids=["fused", "lockstep"])
@pytest.mark.parametrize("wl", CONV_SWEEP_CASES, ids=lambda w: w.name)
def test_conv_forward_fused_sweeps(wl, fused, monkeypatch):
    import paper_2007_07336_amd as M
    if not fused:
        monkeypatch.setenv("MGRIT_NO_SWEEP", "1")
    _announce(f"{wl.name} fused={fused}")
    data = I.generate(wl)
    gp = GpuProblem(wl, data)
    M.mgrit_trace_begin()
    rc, U, hist, it = gp.forward()
    tr = M.mgrit_trace_end()
    assert ("conv_sweep_kernel" in tr) == fused, tr                           # the path under test did run
    Uo, hist_o, it_o = oracle_forward(wl, data)
    assert rel_l2_per_state(U, Uo) <= TOL[wl.dtype]
    assert it == it_o
    for a, b in zip(hist, hist_o):
        assert abs(a - b) <= 1e-3 * max(b, 1e-6)


def test_conv_fused_sweeps_nested_start():
    wl = I.reduced(I.cfg3(2), name="csweep_fp32_c16_6x6_B32_N48_m3_L3_nested", B=32, Himg=6, Wimg=6, N=48, m=3, max_levels=3,
                   lifted_input=False, act=I.TANH)
    _announce(wl.name)
    data = I.generate(wl)
    gp = GpuProblem(wl, data, init=3)
    rc, U, hist, it = gp.forward()
    Uo, hist_o, _ = oracle_forward(wl, data, init=3)
    assert rel_l2_per_state(U, Uo) <= 1e-5


CONV_SWEEP_ADJ_CASES = [
    I.reduced(I.cfg3(2), name="adj_csweep_fp32_c16_7x5_B8_N64_m4_tanh", B=8, Himg=7, Wimg=5, N=64, act=I.TANH),
    I.reduced(I.cfg3(1), name="adj_csweep_fp32_c8_12x12_B8_N66_m4_relu_trailing", B=8, C=8, Himg=12, Wimg=12, N=66,
              lifted_input=False),
    I.reduced(I.cfg3(1), name="adj_csweep_fp32_c16_9x9_B32_N48_m3_L3_rhs", B=32, Himg=9, Wimg=9, N=48, m=3, max_levels=3,
              lifted_input=False, act=I.TANH),
]


@pytest.mark.parametrize("fused", [True, False], ids=["fused", "lockstep"])
@pytest.mark.parametrize("wl", CONV_SWEEP_ADJ_CASES, ids=lambda w: w.name)
def test_conv_adjoint_fused_sweeps(wl, fused, monkeypatch):
    import paper_2007_07336_amd as M
    if not fused:
        monkeypatch.setenv("MGRIT_NO_SWEEP", "1")
    _announce(f"{wl.name} fused={fused}")
    data = I.generate(wl)
    Uo, _, _ = oracle_forward(wl, data, max_iter=2)
    U = Uo.astype(np.float32)
    lamN = np.random.default_rng(9).standard_normal(wl.state_shape).astype(np.float32)
    gp = GpuProblem(wl, data)
    M.mgrit_trace_begin()
    Lam, dW, db, hist, it = gp.adjoint(U, lamN)
    tr = M.mgrit_trace_end()
    assert ("conv_sweep_kernel" in tr) == fused, tr
    Lo, dWo, dbo, hist_o, it_o = oracle_adjoint(wl, data, U, lamN)
    eL, eW, eb = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo), rel_l2_per_state(db, dbo)
    assert eL <= 1e-5 and eW <= 1e-5 and eb <= 1e-5, (eL, eW, eb)


@pytest.mark.parametrize("kind", ["dense", "conv"])
def test_fused_sweeps_repeat_bitwise_and_replay_from_a_hip_graph(kind):
    """The fused sweep launches are deterministic, and a forward + adjoint pair that uses them can be captured
    into a HIP graph and replayed to the same bits."""
    import torch
    import paper_2007_07336_amd as M
    if kind == "dense":
        wl = I.reduced(I.cfg2(2), name="sweep_fp32_q256_B64_N256_graph", q=256, B=64, N=256)
    else:
        wl = I.reduced(I.cfg3(2), name="csweep_fp32_c16_12x12_B16_N64_graph", B=16, Himg=12, Wimg=12, N=64, act=I.TANH)
    _announce(wl.name)
    data = I.generate(wl)
    gp = GpuProblem(wl, data)
    lamN = torch.from_numpy(np.random.default_rng(4).standard_normal(wl.state_shape).astype(np.float32)).cuda()
    Lam = torch.zeros_like(gp.U)
    dW = torch.zeros(gp.W.shape, dtype=torch.float32, device="cuda")
    db = torch.zeros_like(gp.b)
    ws = torch.empty(M.mgrit_adjoint_workspace_bytes(gp.p), dtype=torch.uint8, device="cuda")

    def pair():
        M.mgrit_fas_forward(gp.p, gp.W, gp.b, gp.u0, gp.U, ws, want_hist=False)
        M.mgrit_fas_adjoint(gp.p, gp.W, gp.b, gp.U, lamN, Lam, dW, db, ws, want_hist=False)

    M.mgrit_trace_begin()
    pair()
    tr = M.mgrit_trace_end()
    assert any(k.startswith("dense_sweep_kernel" if kind == "dense" else "conv_sweep_kernel") for k in tr), tr
    torch.cuda.synchronize()
    ref = [t.clone() for t in (gp.U, Lam, dW, db)]
    for t in (gp.U, Lam, dW, db):
        t.zero_()
    pair()
    torch.cuda.synchronize()
    for t, r in zip((gp.U, Lam, dW, db), ref):
        assert torch.equal(t, r)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            pair()
    torch.cuda.synchronize()
    for replay in range(3):
        for t in (gp.U, Lam, dW, db):
            t.fill_(float(replay + 1))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, r in zip((gp.U, Lam, dW, db), ref):
            assert torch.equal(t, r), replay
