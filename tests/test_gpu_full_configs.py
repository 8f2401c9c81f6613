"""GPU parity at the full sizes of the five benchmark workloads, in the launch configuration
bench.py times.  Where the CPU oracle finishes the whole schedule in well under two minutes the
comparison is element by element; for the two large workloads (conv 64ch x 512 layers, dense
q=1024 x 1024 layers with adjoint) the oracle re-computes sampled outputs one by one from the
GPU's own neighbouring values (every F-point equals one layer step of its predecessor after the
closing F-relaxation; every sampled layer gradient is one contraction), and the remaining
properties (residual history decreasing, agreement with serial propagation improving) hold at
any size.
"""
import numpy as np
import pytest

import mgrit_inputs as I
from oracle import mgrit_oracle as O
from tests.gpu_util import GpuProblem, oracle_forward, rel_l2_per_state

pytestmark = pytest.mark.gpu
TOL = {I.FP32: 1e-5, I.BF16: 2e-2}


def _say(msg):
    print(f"\n[case] {msg}", flush=True)


def _rel(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b) / max(np.linalg.norm(b), 1e-300))


def test_cfg2_full_elementwise_and_run_to_tolerance():
    wl = I.cfg2(2)
    _say(wl.name)
    data = I.generate(wl)
    gp = GpuProblem(wl, data)
    _, U, hist, it = gp.forward()
    Uo, hist_o, _ = oracle_forward(wl, data)
    err = rel_l2_per_state(U, Uo)
    assert err <= 1e-5, err
    for a, b in zip(hist, hist_o):
        assert abs(a - b) <= 1e-3 * b, (hist, hist_o)
    # run to RMS residual 1e-6: same number of cycles as the oracle (within one) and the
    # result agrees with serial propagation
    wl_t = I.cfg2(40)
    gp = GpuProblem(wl_t, data, tol=1e-6, norm_kind=1)
    _, Ut, hist_t, it_t = gp.forward()
    _, hist_ot, it_ot = oracle_forward(wl_t, data, tol=1e-6, norm_kind=1)
    assert abs(it_t - it_ot) <= 1 and hist_t[-1] <= 1e-6
    Us = O.serial_forward(data["W"], data["b"], data["u0"], wl.h, wl.layer, wl.act)
    err = rel_l2_per_state(Ut, Us)
    assert err <= 1e-5, err


def test_cfg3_full_elementwise():
    wl = I.cfg3(1)
    _say(wl.name)
    data = I.generate(wl)
    gp = GpuProblem(wl, data)
    _, U, hist, it = gp.forward()
    Uo, hist_o, _ = oracle_forward(wl, data)
    err = rel_l2_per_state(U, Uo)
    assert err <= 1e-5, err
    assert abs(hist[0] - hist_o[0]) <= 1e-3 * hist_o[0], (hist, hist_o)


def test_cfg3_full_adjoint_elementwise():
    """Adjoint solve and parameter gradient (layers split into partial sums) at full size, element by element.

    ReLU' is a 0/1 decision on the sign of z = A u + b, and one flipped decision changes a gradient entry by
    O(1), so both sides must take every decision identically.  The weights, biases and the states to linearise
    about are therefore put on coarse binary grids (weights in steps of 2^-7 below 1/2, states in steps of 2^-5
    below 2, biases in steps of 2^-12): every product and every partial sum of the 144 terms of z is then exact
    in float32 in any summation order, so z is the same number on both sides."""
    wl = I.cfg3(1)
    _say(wl.name + " adjoint + gradient")
    data = dict(I.generate(wl))
    data["W"] = (np.clip(np.round(data["W"] * 128.0), -63, 63) / 128.0).astype(np.float32)
    data["b"] = (np.round(data["b"] * 4096.0) / 4096.0).astype(np.float32)
    Uo, _, _ = oracle_forward(wl, data)
    U = (np.clip(np.round(Uo * 32.0), -63, 63) / 32.0).astype(np.float32)
    del Uo
    rng = np.random.default_rng(21)
    lamN = (rng.standard_normal(wl.state_shape) / wl.B).astype(np.float32)
    gp = GpuProblem(wl, data)
    Lam, dW, db, hist, it = gp.adjoint(U, lamN)
    Lo, dWo, dbo, hist_o, _ = O.fas_adjoint(data["W"], data["b"], U, lamN, wl.h, wl.m, wl.max_levels, wl.min_coarse,
                                            wl.relax, wl.max_iter, wl.layer, wl.act)
    eL, eW, eb = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo), rel_l2_per_state(db, dbo)
    print(f"cfg3 adjoint: Lam {eL:.3e}  dW {eW:.3e}  db {eb:.3e}", flush=True)
    assert eL <= 1e-5 and eW <= 1e-5 and eb <= 1e-5, (eL, eW, eb)


def test_cfg3_full_adjoint_raw_inputs():
    """The same at full size on the raw random inputs (nothing put on a grid).  Both sides now take a ReLU' decision
    on their own value of z, and the two values differ by float32 rounding (z is a sum of 144 terms of unit scale),
    so a decision can differ where |z| is of that size.  One differing decision moves one of the 802 816 entries of a
    layer's G = ReLU'(z) .* Lam, i.e. that layer's gradient by about 1 / sqrt(802 816) = 1.1e-3 of its norm, and
    reaches the adjoint states behind it scaled by h.  So: the adjoint states agree to 1e-4; a layer without a
    pre-activation within 1e-5 of zero agrees to 1e-4 in its gradient (what arrives from other layers' decisions);
    a layer with k such pre-activations may be off by 1.2e-3 for each of them."""
    wl = I.cfg3(1)
    _say(wl.name + " adjoint + gradient, raw inputs")
    data = I.generate(wl)
    Uo, _, _ = oracle_forward(wl, data)
    U = Uo.astype(np.float32)
    del Uo
    rng = np.random.default_rng(22)
    lamN = (rng.standard_normal(wl.state_shape) / wl.B).astype(np.float32)
    gp = GpuProblem(wl, data)
    Lam, dW, db, hist, it = gp.adjoint(U, lamN)
    Lo, dWo, dbo, hist_o, _ = O.fas_adjoint(data["W"], data["b"], U, lamN, wl.h, wl.m, wl.max_levels, wl.min_coarse,
                                            wl.relax, wl.max_iter, wl.layer, wl.act)
    eL = rel_l2_per_state(Lam, Lo)
    assert eL <= 1e-4, eL
    worst, total_near = 0.0, 0
    for n in range(wl.N):
        z = O.affine(U[n].astype(np.float64), data["W"][n].astype(np.float64), data["b"][n].astype(np.float64), wl.layer)
        near = int((np.abs(z) < 1e-5).sum())
        total_near += near
        eW, eb = _rel(dW[n], dWo[n]), _rel(db[n], dbo[n])
        worst = max(worst, eW, eb)
        assert max(eW, eb) <= 1e-4 + 1.2e-3 * near, (n, eW, eb, near)
    print(f"cfg3 adjoint, raw inputs: Lam {eL:.3e}, worst layer gradient {worst:.3e}; {total_near} of "
          f"{wl.N * U[0].size} pre-activations within 1e-5 of zero", flush=True)


def _sampled_f_point_checks(wl, data, U, rng, n_samples):
    """Every F-point j (j % m != 0) equals one layer step of point j-1 after the closing F-relaxation."""
    W64 = data["W"]
    worst = 0.0
    js = [j for j in rng.choice(np.arange(1, wl.N + 1), size=4 * n_samples, replace=False) if j % wl.m != 0]
    for j in js[:n_samples]:
        ref = O.step(U[j - 1].astype(np.float64), W64[j - 1].astype(np.float64), data["b"][j - 1].astype(np.float64),
                     wl.h, wl.layer, wl.act)
        inc_ref = ref - U[j - 1]
        inc_got = U[j].astype(np.float64) - U[j - 1]
        worst = max(worst, _rel(inc_got, inc_ref) if wl.dtype == I.BF16 else _rel(U[j], ref))
    return worst


def test_cfg4_full_sampled():
    wl = I.cfg4(2)
    _say(wl.name)
    data = I.generate(wl)
    gp = GpuProblem(wl, data)
    _, U, hist, it = gp.forward()
    assert it == 2 and hist[1] < hist[0]
    rng = np.random.default_rng(11)
    # increments h*F of sampled F-points, recomputed by the oracle from the GPU's own predecessor
    worst = _sampled_f_point_checks(wl, data, U, rng, 8)
    assert worst <= 2e-2, worst
    # the first coarse interval is exact after the first cycle: compare with serial propagation there
    Us = O.serial_forward(data["W"][:wl.m], data["b"][:wl.m], data["u0"], wl.h, wl.layer, wl.act)
    err = rel_l2_per_state(U[:wl.m + 1], Us)
    assert err <= 2e-2, err
    inc = rel_l2_per_state(U[1:wl.m + 1] - U[0], Us[1:] - Us[0])
    assert inc <= 2e-2, inc
    del U


def test_cfg4_full_adjoint_gradient_sampled():
    """Adjoint solve and parameter gradient of the large conv workload (one workgroup per layer, no partial
    sums): sampled adjoint F-points and sampled layer gradients, recomputed by the oracle from the GPU's own
    neighbouring values."""
    wl = I.cfg4(2)
    _say(wl.name + " adjoint + gradient")
    data = I.generate(wl)
    gp = GpuProblem(wl, data)
    _, U, _, _ = gp.forward()
    # ReLU' is a 0/1 decision on the sign of z: both sides take it from the same bf16-representable states
    U = I.round_to_bf16(U)
    rng = np.random.default_rng(22)
    lamN = (rng.standard_normal(wl.state_shape) / wl.B).astype(np.float32)
    Lam, dW, db, hist, it = gp.adjoint(U, lamN)
    assert it == 2 and hist[1] < hist[0]
    same = bool(np.array_equal(Lam[wl.N], lamN))
    assert same
    W, b = data["W"], data["b"]
    for n in rng.choice(np.arange(wl.N), size=4, replace=False):
        Wn, bn, Un = W[n].astype(np.float64), b[n].astype(np.float64), U[n].astype(np.float64)
        if n % wl.m != 0:
            ref = O.adjoint_step(Lam[n + 1].astype(np.float64), Un, Wn, bn, wl.h, wl.layer, wl.act)
            e = _rel(Lam[n].astype(np.float64) - Lam[n + 1], ref - Lam[n + 1])
            assert e <= 2e-2, (n, e)
        G = O.act_prime(O.affine(Un, Wn, bn, wl.layer), wl.act) * Lam[n + 1].astype(np.float64)
        gW, gb = O.weight_grad(G, Un, wl.layer)
        eW, eb = _rel(dW[n], wl.h * gW), _rel(db[n], wl.h * gb)
        print(f"cfg4 layer {n}: dW {eW:.3e} db {eb:.3e}", flush=True)
        assert eW <= 2e-2 and eb <= 2e-2, (n, eW, eb)
    del U, Lam, dW


@pytest.fixture(scope="module")
def cfg5_data():
    wl = I.cfg5(1)
    return wl, I.generate(wl)


def test_cfg5_full_forward_elementwise(cfg5_data):
    wl, data = cfg5_data
    _say(wl.name + " forward, 1 cycle")
    gp = GpuProblem(wl, data)
    _, U, hist, it = gp.forward()
    Uo, hist_o, _ = oracle_forward(wl, data)
    err = rel_l2_per_state(U, Uo)
    # the change relative to the initial guess u0 (a much smaller quantity than the state) as a
    # sharper diagnostic of the bf16 operand rounding; looser bound, printed
    err_inc = rel_l2_per_state(U[1:] - U[0], Uo[1:] - Uo[0])
    print(f"cfg5 forward: per-state rel L2 {err:.3e}, per-state increment rel L2 {err_inc:.3e}, "
          f"hist {hist} vs oracle {hist_o}", flush=True)
    assert err <= 2e-2, err
    assert err_inc <= 1e-1, err_inc
    assert abs(hist[0] - hist_o[0]) <= 5e-2 * hist_o[0], (hist, hist_o)


def test_cfg5_full_training_step_sampled(cfg5_data):
    import dataclasses
    wl1, data = cfg5_data
    wl = dataclasses.replace(wl1, max_iter=2)
    _say(wl.name + " forward + adjoint + gradient, 2 cycles")
    gp = GpuProblem(wl, data)
    _, U, hist, it = gp.forward()
    assert it == 2 and hist[1] < hist[0]
    lamN = I.terminal_adjoint(wl, data, U[-1])
    Lam, dW, db, hist_a, it_a = gp.adjoint(U, lamN)
    assert it_a == 2 and hist_a[1] < hist_a[0]
    same = bool(np.array_equal(Lam[wl.N], lamN))
    assert same
    rng = np.random.default_rng(12)
    worst = _sampled_f_point_checks(wl, data, U, rng, 6)
    assert worst <= 2e-2, worst
    W, b = data["W"], data["b"]
    for n in rng.choice(np.arange(wl.N), size=6, replace=False):
        Wn, bn = W[n].astype(np.float64), b[n].astype(np.float64)
        Un = U[n].astype(np.float64)
        if n % wl.m != 0:      # F-point: one adjoint step of its successor after the closing F-relaxation
            ref = O.adjoint_step(Lam[n + 1].astype(np.float64), Un, Wn, bn, wl.h, wl.layer, wl.act)
            e = _rel(Lam[n].astype(np.float64) - Lam[n + 1], ref - Lam[n + 1])
            assert e <= 2e-2, (n, e)
        G = O.act_prime(O.affine(Un, Wn, bn, wl.layer), wl.act) * Lam[n + 1].astype(np.float64)
        gW, gb = O.weight_grad(G, Un, wl.layer)
        eW, eb = _rel(dW[n], wl.h * gW), _rel(db[n], wl.h * gb)
        assert eW <= 2e-2 and eb <= 2e-2, (n, eW, eb)


def test_cfg5_full_adjoint_elementwise(cfg5_data):
    """Adjoint solve (1 cycle) and parameter gradient at full size, element by element, linearised about the
    oracle's own one-cycle forward iterate."""
    wl, data = cfg5_data
    _say(wl.name + " adjoint + gradient, 1 cycle, element-wise")
    Uo, _, _ = oracle_forward(wl, data)
    U = Uo.astype(np.float32)
    del Uo
    lamN = I.terminal_adjoint(wl, data, U[-1])
    gp = GpuProblem(wl, data)
    Lam, dW, db, hist, it = gp.adjoint(U, lamN)
    Lo, dWo, dbo, hist_o, _ = O.fas_adjoint(data["W"], data["b"], U, lamN, wl.h, wl.m, wl.max_levels, wl.min_coarse,
                                            wl.relax, wl.max_iter, wl.layer, wl.act)
    eL, eW, eb = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo), rel_l2_per_state(db, dbo)
    print(f"cfg5 adjoint: Lam {eL:.3e}  dW {eW:.3e}  db {eb:.3e}  hist {hist} vs {hist_o}", flush=True)
    assert eL <= 2e-2 and eW <= 2e-2 and eb <= 2e-2, (eL, eW, eb)


# ------------------------------------------------------------------------------------------------
# The two large workloads through their WHOLE hierarchy against the full oracle (Alg. 1 steps 1-6 on
# every level: relaxation, residual, injection, coarse right-hand side, recursive / serial coarse
# solve, correction), at the workload's own N, m, level count, relaxation and operand type, two
# cycles, forward and adjoint with the parameter gradient.  Only the batch is cut so that the
# float64 oracle finishes in about a minute; a layer step treats every sample alike, so the level
# schedule, index maps and kernels at the fine level are those of the full batch.
# ------------------------------------------------------------------------------------------------
def _full_hierarchy_case(wl, lam_from_head, data=None):
    data = I.generate(wl) if data is None else data
    gp = GpuProblem(wl, data)
    sizes, _ = gp.M.mgrit_level_map(gp.p)
    _say(f"{wl.name}: levels {sizes}, batch {wl.B}, {wl.max_iter} cycles, forward")
    _, U, hist, it = gp.forward()
    Uo, hist_o, it_o = oracle_forward(wl, data)
    assert it == it_o == wl.max_iter
    err = rel_l2_per_state(U, Uo)
    err_inc = rel_l2_per_state(U[1:] - U[0], Uo[1:] - Uo[0])
    print(f"{wl.name} forward: per-state rel L2 {err:.3e}, increment rel L2 {err_inc:.3e}, "
          f"hist {hist} vs oracle {hist_o}", flush=True)
    assert err <= TOL[wl.dtype], err
    assert err_inc <= 1e-1, err_inc
    for a, b in zip(hist, hist_o):
        assert abs(a - b) <= 5e-2 * b, (hist, hist_o)
    # adjoint about bf16-representable states (both sides then take every act' decision from the same
    # operand values, the kernel's), two cycles, and the parameter gradient of every layer
    _say(f"{wl.name}: adjoint + gradient")
    Ulin = I.round_to_bf16(Uo.astype(np.float32))
    del Uo, U
    if lam_from_head:
        lamN = I.terminal_adjoint(wl, data, Ulin[-1])
    else:
        lamN = (np.random.default_rng(23).standard_normal(wl.state_shape) / wl.B).astype(np.float32)
    Lam, dW, db, hist_a, it_a = gp.adjoint(Ulin, lamN)
    Lo, dWo, dbo, hist_ao, _ = O.fas_adjoint(data["W"], data["b"], Ulin, lamN, wl.h, wl.m, wl.max_levels,
                                              wl.min_coarse, wl.relax, wl.max_iter, wl.layer, wl.act)
    eL, eW, eb = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo), rel_l2_per_state(db, dbo)
    print(f"{wl.name} adjoint: Lam {eL:.3e}  dW {eW:.3e}  db {eb:.3e}  hist {hist_a} vs {hist_ao}", flush=True)
    assert it_a == wl.max_iter
    assert eL <= TOL[wl.dtype] and eW <= TOL[wl.dtype] and eb <= TOL[wl.dtype], (eL, eW, eb)
    for a, b in zip(hist_a, hist_ao):
        assert abs(a - b) <= 5e-2 * b, (hist_a, hist_ao)


def test_cfg4_whole_hierarchy_two_cycles_against_the_oracle():
    """512 / 64 / 8 layers, m = 8, FCF, bf16 operands, 64 channels on 32x32 images; batch 2 of 32."""
    _full_hierarchy_case(I.reduced(I.cfg4(2), name="cfg4_hierarchy_B2", B=2), lam_from_head=False)


def test_cfg5_whole_hierarchy_two_cycles_against_the_oracle(cfg5_data):
    """1024 / 64 / 4 layers, m = 16, FCF, bf16 operands, width 1024, softmax head; the first 32 of the 256 samples
    (parameters and head are those of the full workload, drawn once for this module)."""
    _, full = cfg5_data
    data = {"W": full["W"], "b": full["b"], "u0": np.ascontiguousarray(full["u0"][:32]), "W_o": full["W_o"],
            "labels": full["labels"][:32]}
    _full_hierarchy_case(I.reduced(I.cfg5(2), name="cfg5_hierarchy_B32", B=32), lam_from_head=True, data=data)
