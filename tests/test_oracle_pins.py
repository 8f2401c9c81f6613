"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test checks the oracle against something that is not the oracle: a closed form, an
invariant of the method, a dense linear-algebra construction, an independent float64
library routine (torch CPU), finite differences, or a scalar brute-force re-derivation.
"""
import math

import numpy as np
import pytest
import torch

from oracle import mgrit_oracle as O

DENSE, CONV = O.DENSE, O.CONV
TANH, RELU, IDENT = O.TANH, O.RELU, O.IDENT


def _dense_problem(rng, N, q, B, bias=True, scale=1.0):
    W = rng.standard_normal((N, q, q)) * scale / math.sqrt(q)
    b = rng.standard_normal((N, q)) * 0.3 if bias else np.zeros((N, q))
    u0 = rng.standard_normal((B, q))
    return W, b, u0


def _conv_problem(rng, N, C, B, H, Wd):
    K = rng.standard_normal((N, C, 3, 3, C)) * math.sqrt(2.0 / (9 * C))
    b = rng.standard_normal((N, C)) * 0.3
    u0 = rng.standard_normal((B, H, Wd, C))
    return K, b, u0


# ---------------------------------------------------------------------------------------
# Layer step against an independent float64 library routine (Sec. II, Eq. (1))
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("kind", [TANH, RELU])
def test_dense_step_matches_torch(kind):
    rng = np.random.default_rng(1)
    W, b, u0 = _dense_problem(rng, 1, 7, 5)
    got = O.step(u0, W[0], b[0], 0.37, DENSE, kind)
    z = torch.nn.functional.linear(torch.from_numpy(u0), torch.from_numpy(W[0]), torch.from_numpy(b[0]))
    f = torch.tanh(z) if kind == TANH else torch.relu(z)
    ref = torch.from_numpy(u0) + 0.37 * f
    np.testing.assert_allclose(got, ref.numpy(), rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("kind", [TANH, RELU])
def test_conv_step_matches_torch_conv2d(kind):
    rng = np.random.default_rng(2)
    K, b, u0 = _conv_problem(rng, 1, 3, 2, 5, 6)      # non-square image, C_in = C_out = 3
    got = O.step(u0, K[0], b[0], 0.21, CONV, kind)
    x = torch.from_numpy(u0).permute(0, 3, 1, 2)        # NCHW
    w = torch.from_numpy(K[0]).permute(0, 3, 1, 2)      # [Co, Ci, 3, 3]
    z = torch.nn.functional.conv2d(x, w, torch.from_numpy(b[0]), padding=1)
    f = torch.tanh(z) if kind == TANH else torch.relu(z)
    ref = (x + 0.21 * f).permute(0, 2, 3, 1)
    np.testing.assert_allclose(got, ref.numpy(), rtol=1e-13, atol=1e-13)


def test_conv_affine_brute_force_asymmetric_kernel():
    """Zero padding, cross-correlation orientation and the [Co,3,3,Ci] layout by explicit loops."""
    rng = np.random.default_rng(3)
    Co, Ci, H, Wd = 2, 3, 4, 3
    K = rng.standard_normal((Co, 3, 3, Ci))
    b = rng.standard_normal(Co)
    u = rng.standard_normal((1, H, Wd, Ci))
    z = O.affine(u, K, b, CONV)
    for y in range(H):
        for x in range(Wd):
            for o in range(Co):
                s = b[o]
                for dy in range(3):
                    for dx in range(3):
                        yy, xx = y + dy - 1, x + dx - 1
                        if 0 <= yy < H and 0 <= xx < Wd:
                            s += float(K[o, dy, dx, :] @ u[0, yy, xx, :])
                assert abs(z[0, y, x, o] - s) < 1e-12


# ---------------------------------------------------------------------------------------
# Linear F: closed-form propagator
# ---------------------------------------------------------------------------------------
def test_linear_diagonal_closed_form():
    N, q, h = 20, 4, 0.05
    lam = np.array([-1.0, 0.5, 2.0, -3.0])
    W = np.tile(np.diag(lam), (N, 1, 1))
    b = np.zeros((N, q))
    u0 = np.array([[1.0, -2.0, 0.5, 3.0]])
    U = O.serial_forward(W, b, u0, h, DENSE, IDENT)
    for n in range(N + 1):
        np.testing.assert_allclose(U[n], u0 * (1 + h * lam) ** n, rtol=1e-13)


def test_linear_product_of_propagators():
    rng = np.random.default_rng(4)
    N, q, h = 6, 3, 0.2
    W, b, u0 = _dense_problem(rng, N, q, 2, bias=False)
    U = O.serial_forward(W, b, u0, h, DENSE, IDENT)
    P = np.eye(q)
    for n in range(N):
        P = (np.eye(q) + h * W[n]) @ P
    np.testing.assert_allclose(U[N], u0 @ P.T, rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------------------------------
# Two-level exactness (Sec. III-C, Alg. 1): with F-relaxation the first k coarse intervals
# are exact after k cycles, for any initial guess; FCF advances two intervals per cycle.
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("N", [12, 13, 14])            # 13, 14: trailing F-points behind the last C-point
@pytest.mark.parametrize("layer", [DENSE, CONV])
@pytest.mark.parametrize("relax,per_cycle", [(O.RELAX_F, 1), (O.RELAX_FCF, 2)])
def test_two_level_exact_after_enough_cycles(layer, relax, per_cycle, N):
    rng = np.random.default_rng(5)
    m = 3
    h = 1.0 / N
    if layer == DENSE:
        W, b, u0 = _dense_problem(rng, N, 5, 3, scale=2.0)
    else:
        W, b, u0 = _conv_problem(rng, N, 2, 2, 4, 3)
    Us = O.serial_forward(W, b, u0, h, layer, TANH)
    Uinit = rng.standard_normal(Us.shape)
    for k in range(1, N // m + 1):
        U, hist, it = O.fas_forward(W, b, u0, h, m, 2, 1, relax, k, layer, TANH, init=2, U_init=Uinit)
        assert it == k and len(hist) == k
        exact_upto = min(N, (per_cycle * k + 1) * m - 1)     # all points of the exact intervals
        err = np.abs(U[:exact_upto + 1] - Us[:exact_upto + 1]).max()
        assert err < 1e-12, (k, err)
        if (per_cycle * k + 1) * m <= N:                     # and the rest is NOT yet exact
            assert np.abs(U[-1] - Us[-1]).max() > 1e-8
    assert np.abs(U - Us).max() < 1e-12


def test_config1_shape_is_exact_after_four_cycles():
    """N=16, m=4, two levels, F-relaxation, 4 cycles reproduces serial propagation."""
    rng = np.random.default_rng(0)
    W, b, u0 = _dense_problem(rng, 16, 8, 4)
    Us = O.serial_forward(W, b, u0, 1 / 16, DENSE, TANH)
    U, hist, _ = O.fas_forward(W, b, u0, 1 / 16, 4, 2, 1, O.RELAX_F, 4, DENSE, TANH)
    assert np.abs(U - Us).max() < 1e-13
    U3, _, _ = O.fas_forward(W, b, u0, 1 / 16, 4, 2, 1, O.RELAX_F, 3, DENSE, TANH)
    assert np.abs(U3 - Us).max() > 1e-9


# ---------------------------------------------------------------------------------------
# Fixed point (Sec. III-A): at the exact solution the residual vanishes and nothing changes
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("levels", [2, 3])
@pytest.mark.parametrize("relax", [O.RELAX_F, O.RELAX_FCF])
def test_fixed_point(levels, relax):
    rng = np.random.default_rng(6)
    N, m = 16, 2
    W, b, u0 = _dense_problem(rng, N, 4, 2, scale=2.0)
    Us = O.serial_forward(W, b, u0, 1 / N, DENSE, RELU)
    U, hist, _ = O.fas_forward(W, b, u0, 1 / N, m, levels, 1, relax, 2, DENSE, RELU, init=2, U_init=Us)
    assert max(hist) < 1e-13
    assert np.abs(U - Us).max() < 1e-13


# ---------------------------------------------------------------------------------------
# Linear F: one two-level FAS cycle equals the textbook linear two-grid correction scheme
# assembled as dense matrices (Sec. III-A, Eq. (9)-(11))
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,m", [(8, 2), (9, 2), (11, 3), (7, 4)])   # the last three end in F-points
@pytest.mark.parametrize("relax", [O.RELAX_F, O.RELAX_FCF])
def test_linear_two_level_equals_dense_two_grid(relax, N, m):
    rng = np.random.default_rng(7)
    q, h = 2, 0.3
    W, b, u0 = _dense_problem(rng, N, q, 1, bias=False, scale=1.5)
    n = (N + 1) * q
    Phi = [np.eye(q) + h * W[k] for k in range(N)]
    A = np.eye(n)
    for k in range(N):
        A[(k + 1) * q:(k + 2) * q, k * q:(k + 1) * q] = -Phi[k]
    f = np.zeros(n)
    f[:q] = u0[0]
    Nc = N // m
    AH = np.eye((Nc + 1) * q)
    for i in range(Nc):
        AH[(i + 1) * q:(i + 2) * q, i * q:(i + 1) * q] = -(np.eye(q) + m * h * W[i * m])
    cidx = np.concatenate([np.arange(i * m * q, i * m * q + q) for i in range(Nc + 1)])

    Uinit = rng.standard_normal((N + 1, 1, q))
    x = Uinit.reshape(-1).copy()
    x[:q] = u0[0]

    def f_relax(x):                       # exact solve of the F-rows given the C-values
        x = x.copy()
        for j in range(1, N + 1):
            if j % m:                     # every point that is not a multiple of m is an F-point
                x[j * q:(j + 1) * q] = Phi[j - 1] @ x[(j - 1) * q:j * q]
        return x

    def c_relax(x):
        x = x.copy()
        for i in range(1, Nc + 1):
            j = i * m
            x[j * q:(j + 1) * q] = Phi[j - 1] @ x[(j - 1) * q:j * q]
        return x

    x = f_relax(x)
    if relax == O.RELAX_FCF:
        x = f_relax(c_relax(x))
    r = f - A @ x
    rnorm = np.linalg.norm(r[cidx])
    assert np.abs(np.delete(r, cidx)).max() < 1e-13        # F-rows have zero residual
    delta = np.linalg.solve(AH, r[cidx])                      # L_H dU_H = I r_h
    x[cidx] += delta                                          # u += I_H^h dU_H (C-points)
    x = f_relax(x)

    U, hist, _ = O.fas_forward(W, b, u0, h, m, 2, 1, relax, 1, DENSE, IDENT, init=2, U_init=Uinit)
    np.testing.assert_allclose(U.reshape(-1), x, rtol=1e-11, atol=1e-12)
    assert abs(hist[0] - rnorm) < 1e-12 * max(1.0, rnorm)


@pytest.mark.parametrize("relax", [O.RELAX_F, O.RELAX_FCF])
def test_linear_three_level_equals_dense_three_grid(relax):
    """A multilevel iterate at a fixed cycle count: for linear F one three-level V-cycle equals the three-grid
    correction scheme assembled from dense matrices -- relax, restrict the residual by injection, solve the
    level-1 correction equation approximately by ONE two-grid cycle from a zero guess (relax, restrict, exact
    solve on level 2, correct, F-relax), correct, F-relax (Sec. III-A applied recursively)."""
    rng = np.random.default_rng(17)
    N, m, q, h = 16, 2, 2, 0.15          # 4 intervals on level 1: one FCF cycle there is not yet exact
    W, b, u0 = _dense_problem(rng, N, q, 1, bias=False, scale=1.5)

    def system(steps, stride, hs):        # block bidiagonal L with -(I + hs W[j * stride]) below the diagonal
        Phi = [np.eye(q) + hs * W[j * stride] for j in range(steps)]
        A = np.eye((steps + 1) * q)
        for j in range(steps):
            A[(j + 1) * q:(j + 2) * q, j * q:(j + 1) * q] = -Phi[j]
        return A, Phi

    A0, Phi0 = system(N, 1, h)
    A1, Phi1 = system(N // m, m, m * h)
    A2, _ = system(N // m // m, m * m, m * m * h)

    def blk(j):
        return slice(j * q, (j + 1) * q)

    def cidx(steps):                      # entries of the C-points 0, m, 2m, ... of a level with `steps` steps
        return np.concatenate([np.arange(i * m * q, i * m * q + q) for i in range(steps // m + 1)])

    def relax_level(x, rhs, Phi, steps, kind):
        def f_rel(x):
            x = x.copy()
            for i in range(steps // m):
                for k in range(1, m):
                    j = i * m + k
                    x[blk(j)] = Phi[j - 1] @ x[blk(j - 1)] + rhs[blk(j)]
            return x

        def c_rel(x):
            x = x.copy()
            for i in range(1, steps // m + 1):
                j = i * m
                x[blk(j)] = Phi[j - 1] @ x[blk(j - 1)] + rhs[blk(j)]
            return x
        x = f_rel(x)
        if kind == O.RELAX_FCF:
            x = f_rel(c_rel(x))
        return x

    f = np.zeros((N + 1) * q)
    f[:q] = u0[0]
    Uinit = rng.standard_normal((N + 1, 1, q))
    x = Uinit.reshape(-1).copy()
    x[:q] = u0[0]
    x = relax_level(x, f, Phi0, N, relax)
    r0 = (f - A0 @ x)[cidx(N)]                                   # level-1 right-hand side of the correction equation
    d1 = relax_level(np.zeros_like(r0), r0, Phi1, N // m, relax)  # zero guess; its point-0 row: d1[0] = r0[0] = 0
    r1 = (r0 - A1 @ d1)[cidx(N // m)]
    d1[cidx(N // m)] += np.linalg.solve(A2, r1)
    d1 = relax_level(d1, r0, Phi1, N // m, O.RELAX_F)
    x[cidx(N)] += d1
    x = relax_level(x, f, Phi0, N, O.RELAX_F)

    U, hist, _ = O.fas_forward(W, b, u0, h, m, 3, 1, relax, 1, DENSE, IDENT, init=2, U_init=Uinit)
    np.testing.assert_allclose(U.reshape(-1), x, rtol=1e-11, atol=1e-12)
    assert abs(hist[0] - np.linalg.norm(r0)) < 1e-12 * max(1.0, np.linalg.norm(r0))
    # and it is a different iterate from the two-level one (the pin would not notice a skipped level otherwise)
    U2, _, _ = O.fas_forward(W, b, u0, h, m, 2, 1, relax, 1, DENSE, IDENT, init=2, U_init=Uinit)
    assert np.abs(U2 - U).max() > 1e-6


# ---------------------------------------------------------------------------------------
# Brute force on a tiny nonlinear scalar instance: an independent pure-Python evaluation of the
# system rows checks the coarse equation L_H(V) = L_H(Ubar) + R_H and the residual norm
# ---------------------------------------------------------------------------------------
def test_scalar_brute_force_coarse_equation_and_norm():
    rng = np.random.default_rng(8)
    N, m, h = 8, 2, 0.25
    w = rng.standard_normal(N) * 1.5
    bb = rng.standard_normal(N) * 0.5
    y0 = 0.7
    x = list(rng.standard_normal(N + 1))
    x[0] = y0

    def F(n, u):
        return math.tanh(w[n] * u + bb[n])

    # F-relaxation by hand
    for i in range(N // m):
        for k in range(1, m):
            j = i * m + k
            x[j] = x[j - 1] + h * F(j - 1, x[j - 1])
    # rows of f_h - L_h(x)
    R = [y0 - x[0]] + [-(x[n] - x[n - 1] - h * F(n - 1, x[n - 1])) for n in range(1, N + 1)]
    Nc = N // m
    ubar = [x[i * m] for i in range(Nc + 1)]
    H = m * h
    LH_ubar = [ubar[0]] + [ubar[i] - ubar[i - 1] - H * F((i - 1) * m, ubar[i - 1]) for i in range(1, Nc + 1)]
    S = [LH_ubar[i] + R[i * m] for i in range(Nc + 1)]

    W = w.reshape(N, 1, 1)
    b = bb.reshape(N, 1)
    u0 = np.array([[y0]])
    Uinit = np.array(x).reshape(N + 1, 1, 1)
    # the hand-relaxed x is a fixed point of the oracle's opening F-relaxation, so the cycle
    # sees exactly this iterate
    U, hist, _ = O.fas_forward(W, b, u0, h, m, 2, 1, O.RELAX_F, 1, DENSE, TANH, init=2, U_init=Uinit)
    V = [float(U[i * m, 0, 0]) for i in range(Nc + 1)]
    LH_V = [V[0]] + [V[i] - V[i - 1] - H * F((i - 1) * m, V[i - 1]) for i in range(1, Nc + 1)]
    for i in range(Nc + 1):
        assert abs(LH_V[i] - S[i]) < 1e-13, i
    assert abs(hist[0] - math.sqrt(sum(R[i * m] ** 2 for i in range(Nc + 1)))) < 1e-13
    # all-points residual norm of an arbitrary iterate
    xr = list(rng.standard_normal(N + 1))
    Rall = [y0 - xr[0]] + [-(xr[n] - xr[n - 1] - h * F(n - 1, xr[n - 1])) for n in range(1, N + 1)]
    got = O.residual_norm(W, b, u0, np.array(xr).reshape(N + 1, 1, 1), h, DENSE, TANH)
    assert abs(got - math.sqrt(sum(r * r for r in Rall))) < 1e-13
    got_rms = O.residual_norm(W, b, u0, np.array(xr).reshape(N + 1, 1, 1), h, DENSE, TANH, norm_kind=1)
    assert abs(got_rms - math.sqrt(sum(r * r for r in Rall) / (N + 1))) < 1e-13


def test_in_cycle_rms_history_brute_force():
    """The residual history with the RMS norm (Alg. 1 step 6; Sec. IV-A reports the L2 norm of R_h) is
    sqrt(sum of R^2 over the fine C-points / number of summed entries), the number of entries being
    (N_1 + 1) * batch * width -- written out here with pure-Python loops over every sample and feature,
    for a two-level and a three-level hierarchy (the count is the fine level's C-points in both), forward
    and adjoint.  A divisor that counted all N + 1 points, forgot point 0, or forgot the batch or the
    width fails."""
    rng = np.random.default_rng(81)
    N, m, h, B, q = 12, 2, 0.2, 3, 2
    W = rng.standard_normal((N, q, q))
    b = rng.standard_normal((N, q)) * 0.5
    u0 = rng.standard_normal((B, q))
    x = rng.standard_normal((N + 1, B, q))
    x[0] = u0

    def phi(n, u):          # one sample: u + h tanh(W_n u + b_n), element by element
        out = []
        for o in range(q):
            z = b[n][o]
            for i in range(q):
                z += W[n][o][i] * u[i]
            out.append(u[o] + h * math.tanh(z))
        return out

    # F-relaxation by hand, then the C-point rows of f_h - L_h(x)
    xs = [[list(x[j][r]) for r in range(B)] for j in range(N + 1)]
    for i in range(N // m):
        for k in range(1, m):
            j = i * m + k
            for r in range(B):
                xs[j][r] = phi(j - 1, xs[j - 1][r])
    ssq, entries = 0.0, 0
    for j in range(0, N + 1, m):
        for r in range(B):
            row = [u0[r][o] - xs[0][r][o] for o in range(q)] if j == 0 else \
                  [p - c for p, c in zip(phi(j - 1, xs[j - 1][r]), xs[j][r])]
            for v in row:
                ssq += v * v
                entries += 1
    assert entries == 7 * 3 * 2                       # (N/m + 1) C-points x batch x width
    Uinit = np.array(xs)
    for levels in (2, 3):                             # 12/6 and 12/6/3: the same fine C-points either way
        _, hist, _ = O.fas_forward(W, b, u0, h, m, levels, 1, O.RELAX_F, 2, DENSE, TANH, init=2, U_init=Uinit,
                                   norm_kind=1)
        assert abs(hist[0] - math.sqrt(ssq / 42.0)) < 1e-13, (levels, hist[0])
        _, hist_l2, _ = O.fas_forward(W, b, u0, h, m, levels, 1, O.RELAX_F, 2, DENSE, TANH, init=2, U_init=Uinit)
        assert abs(hist_l2[0] - math.sqrt(ssq)) < 1e-13
        for a, c in zip(hist, hist_l2):               # every cycle's entry carries the same divisor
            assert abs(a - c / math.sqrt(42.0)) < 1e-14
    # adjoint: the same count on the reversed axis (N = 13, m = 3: C-points 13, 10, 7, 4, 1 -> 5 of them)
    N2, m2 = 13, 3
    W2 = rng.standard_normal((N2, q, q))
    b2 = rng.standard_normal((N2, q)) * 0.5
    U2 = rng.standard_normal((N2 + 1, B, q))
    lamN = rng.standard_normal((B, q))
    _, _, _, ha, _ = O.fas_adjoint(W2, b2, U2, lamN, h, m2, 2, 1, O.RELAX_FCF, 2, DENSE, TANH, norm_kind=1)
    _, _, _, ha2, _ = O.fas_adjoint(W2, b2, U2, lamN, h, m2, 2, 1, O.RELAX_FCF, 2, DENSE, TANH, norm_kind=0)
    for a, c in zip(ha, ha2):
        assert abs(a - c / math.sqrt(5 * 3 * 2)) < 1e-14


# ---------------------------------------------------------------------------------------
# Multilevel: converges to serial propagation, the limit the iteration is defined by
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("layer", [DENSE, CONV])
def test_three_level_converges_to_serial(layer):
    rng = np.random.default_rng(9)
    N, m = 32, 2
    if layer == DENSE:
        W, b, u0 = _dense_problem(rng, N, 6, 3)
    else:
        W, b, u0 = _conv_problem(rng, N, 2, 1, 4, 4)
    Us = O.serial_forward(W, b, u0, 1 / N, layer, TANH)
    U, hist, it = O.fas_forward(W, b, u0, 1 / N, m, 3, 1, O.RELAX_FCF, 30, layer, TANH, tol=1e-13)
    assert it < 30 and hist[-1] <= 1e-13
    assert np.abs(U - Us).max() < 1e-11
    assert all(hist[i + 1] < hist[i] for i in range(len(hist) - 1))


@pytest.mark.parametrize("N,m", [(23, 2), (30, 4), (27, 3), (31, 3)])
def test_three_level_with_trailing_f_points_converges_to_serial_forward_and_adjoint(N, m):
    """Level sizes that are not multiples of m (23 -> 11 -> 5, 30 -> 7 -> 1, 27 -> 9 -> 3, 31 -> 10 -> 3):
    the limit is still serial propagation and its gradient, and a converged solve is a fixed point."""
    rng = np.random.default_rng(90 + N)
    W, b, u0 = _dense_problem(rng, N, 5, 3)
    h = 1.0 / N
    assert O.level_sizes(N, m, 3, 1) == [N, N // m, N // m // m]
    Us = O.serial_forward(W, b, u0, h, DENSE, TANH)
    U, hist, it = O.fas_forward(W, b, u0, h, m, 3, 1, O.RELAX_FCF, 40, DENSE, TANH, tol=1e-13)
    assert it < 40 and np.abs(U - Us).max() < 1e-11
    U2, hist2, _ = O.fas_forward(W, b, u0, h, m, 3, 1, O.RELAX_F, 1, DENSE, TANH, init=2, U_init=Us)
    assert np.abs(U2 - Us).max() < 1e-13 and hist2[0] < 1e-13
    lamN = rng.standard_normal(u0.shape)
    Ls, dWs, dbs = O.serial_backward(W, b, Us, lamN, h, DENSE, TANH)
    Lam, dW, db, hist, it = O.fas_adjoint(W, b, Us, lamN, h, m, 3, 1, O.RELAX_FCF, 40, DENSE, TANH, tol=1e-13)
    assert it < 40
    np.testing.assert_allclose(Lam, Ls, atol=1e-11)
    np.testing.assert_allclose(dW, dWs, atol=1e-11)
    np.testing.assert_allclose(db, dbs, atol=1e-11)


def test_adjoint_two_grid_with_trailing_f_points_equals_dense_two_grid_of_the_reversed_system():
    """Linear layers, N = 7, m = 3: one adjoint cycle is the dense two-grid step for the system
    lam^n - (I + h W^n)^T lam^{n+1} = 0, lam^N given, whose C-points are counted from layer N
    (N, N-m, ...) and whose coarse step over [n, n+m] uses layer n with step m h."""
    rng = np.random.default_rng(77)
    N, m, q, h = 7, 3, 2, 0.3
    W, b, u0 = _dense_problem(rng, N, q, 1, bias=False, scale=1.5)
    U = np.zeros((N + 1, 1, q))
    lamN = rng.standard_normal((1, q))
    n = (N + 1) * q
    PhiT = [(np.eye(q) + h * W[k]).T for k in range(N)]
    A = np.eye(n)                                    # unknowns ordered by fine layer index
    for k in range(N):
        A[k * q:(k + 1) * q, (k + 1) * q:(k + 2) * q] = -PhiT[k]
    f = np.zeros(n)
    f[N * q:] = lamN[0]
    Nc = N // m
    cpts = [N - i * m for i in range(Nc + 1)]        # 7, 4, 1
    AH = np.eye((Nc + 1) * q)                        # coarse unknown i sits at fine point N - i m
    for i in range(Nc):
        lo = N - (i + 1) * m
        AH[(i + 1) * q:(i + 2) * q, i * q:(i + 1) * q] = -(np.eye(q) + m * h * W[lo]).T
    cidx = np.concatenate([np.arange(c * q, c * q + q) for c in cpts])
    Linit = rng.standard_normal((N + 1, 1, q))
    x = Linit.reshape(-1).copy()
    x[N * q:] = lamN[0]

    def f_relax(x):
        x = x.copy()
        for j in range(N - 1, -1, -1):
            if j not in cpts:
                x[j * q:(j + 1) * q] = PhiT[j] @ x[(j + 1) * q:(j + 2) * q]
        return x

    x = f_relax(x)
    r = f - A @ x
    assert np.abs(np.delete(r, cidx)).max() < 1e-13
    x[cidx] += np.linalg.solve(AH, r[cidx])
    x = f_relax(x)
    Lam, dW, db, hist, _ = O.fas_adjoint(W, b, U, lamN, h, m, 2, 1, O.RELAX_F, 1, DENSE, IDENT,
                                         init=2, Lam_init=Linit)
    np.testing.assert_allclose(Lam.reshape(-1), x, rtol=1e-11, atol=1e-12)
    assert abs(hist[0] - np.linalg.norm(r[cidx])) < 1e-12


def test_three_levels_with_coarsest_of_full_depth_equals_two_level():
    """max_levels=3 but min_coarse stops coarsening after one level -> identical to two-level."""
    rng = np.random.default_rng(10)
    N, m = 16, 4
    W, b, u0 = _dense_problem(rng, N, 4, 2)
    a = O.fas_forward(W, b, u0, 1 / N, m, 3, 4, O.RELAX_FCF, 2, DENSE, TANH)
    c = O.fas_forward(W, b, u0, 1 / N, m, 2, 1, O.RELAX_FCF, 2, DENSE, TANH)
    assert np.array_equal(a[0], c[0]) and a[1] == c[1]


def test_single_level_is_serial_propagation():
    rng = np.random.default_rng(11)
    W, b, u0 = _dense_problem(rng, 7, 3, 2)
    U, hist, it = O.fas_forward(W, b, u0, 0.1, 2, 1, 1, O.RELAX_F, 5, DENSE, RELU)
    assert np.array_equal(U, O.serial_forward(W, b, u0, 0.1, DENSE, RELU)) and it == 1


# ---------------------------------------------------------------------------------------
# Serial gradient against finite differences and automatic differentiation
# ---------------------------------------------------------------------------------------
def _loss_np(W, b, u0, h, layer, kind, Cw):
    return float(np.sum(Cw * O.serial_forward(W, b, u0, h, layer, kind)[-1]))


@pytest.mark.parametrize("layer", [DENSE, CONV])
def test_serial_gradient_vs_finite_differences(layer):
    rng = np.random.default_rng(12)
    N, h = 5, 0.2
    if layer == DENSE:
        W, b, u0 = _dense_problem(rng, N, 4, 3, scale=1.5)
    else:
        W, b, u0 = _conv_problem(rng, N, 2, 2, 3, 4)
    Cw = rng.standard_normal(u0.shape)                   # loss = <Cw, u^N>  ->  lam^N = Cw
    U = O.serial_forward(W, b, u0, h, layer, TANH)
    Lam, dW, db = O.serial_backward(W, b, U, Cw, h, layer, TANH)
    eps = 1e-6
    for _ in range(12):
        idx = tuple(rng.integers(0, s) for s in W.shape)
        Wp, Wm = W.copy(), W.copy()
        Wp[idx] += eps
        Wm[idx] -= eps
        fd = (_loss_np(Wp, b, u0, h, layer, TANH, Cw) - _loss_np(Wm, b, u0, h, layer, TANH, Cw)) / (2 * eps)
        assert abs(fd - dW[idx]) <= 1e-6 * max(1.0, abs(fd)), (idx, fd, dW[idx])
    for _ in range(6):
        idx = tuple(rng.integers(0, s) for s in b.shape)
        bp, bm = b.copy(), b.copy()
        bp[idx] += eps
        bm[idx] -= eps
        fd = (_loss_np(W, bp, u0, h, layer, TANH, Cw) - _loss_np(W, bm, u0, h, layer, TANH, Cw)) / (2 * eps)
        assert abs(fd - db[idx]) <= 1e-6 * max(1.0, abs(fd))
    for _ in range(6):                                   # lam^0 = dLoss/du^0
        idx = tuple(rng.integers(0, s) for s in u0.shape)
        up, um = u0.copy(), u0.copy()
        up[idx] += eps
        um[idx] -= eps
        fd = (_loss_np(W, b, up, h, layer, TANH, Cw) - _loss_np(W, b, um, h, layer, TANH, Cw)) / (2 * eps)
        assert abs(fd - Lam[0][idx]) <= 1e-6 * max(1.0, abs(fd))


@pytest.mark.parametrize("layer,kind", [(DENSE, TANH), (DENSE, RELU), (CONV, TANH), (CONV, RELU)])
def test_serial_gradient_vs_autograd(layer, kind):
    rng = np.random.default_rng(13)
    N, h = 4, 0.25
    if layer == DENSE:
        W, b, u0 = _dense_problem(rng, N, 5, 3)
    else:
        W, b, u0 = _conv_problem(rng, N, 3, 2, 4, 5)
    Cw = rng.standard_normal(u0.shape)
    U = O.serial_forward(W, b, u0, h, layer, kind)
    Lam, dW, db = O.serial_backward(W, b, U, Cw, h, layer, kind)
    Wt = torch.tensor(W, requires_grad=True)
    bt = torch.tensor(b, requires_grad=True)
    ut = torch.tensor(u0, requires_grad=True)
    x = ut
    f = torch.tanh if kind == TANH else torch.relu
    for n in range(N):
        if layer == DENSE:
            z = torch.nn.functional.linear(x, Wt[n], bt[n])
        else:
            z = torch.nn.functional.conv2d(x.permute(0, 3, 1, 2), Wt[n].permute(0, 3, 1, 2), bt[n],
                                           padding=1).permute(0, 2, 3, 1)
        x = x + h * f(z)
    (x * torch.tensor(Cw)).sum().backward()
    np.testing.assert_allclose(dW, Wt.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(db, bt.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(Lam[0], ut.grad.numpy(), rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------------------------------
# Adjoint multigrid: mirror of the forward exactness; its limit is the serial gradient
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("N", [12, 13, 14])            # 13, 14: the reversed axis ends in F-points at layer 0
@pytest.mark.parametrize("layer", [DENSE, CONV])
@pytest.mark.parametrize("relax,per_cycle", [(O.RELAX_F, 1), (O.RELAX_FCF, 2)])
def test_adjoint_two_level_exactness(layer, relax, per_cycle, N):
    rng = np.random.default_rng(14)
    m = 3
    h = 1.0 / N
    if layer == DENSE:
        W, b, u0 = _dense_problem(rng, N, 5, 3, scale=2.0)
    else:
        W, b, u0 = _conv_problem(rng, N, 2, 2, 4, 3)
    U = O.serial_forward(W, b, u0, h, layer, TANH)
    U += 0.05 * rng.standard_normal(U.shape)             # linearise about NON-converged states
    lamN = rng.standard_normal(u0.shape)
    Ls, dWs, dbs = O.serial_backward(W, b, U, lamN, h, layer, TANH)
    Linit = rng.standard_normal(U.shape)
    for k in range(1, N // m + 1):
        Lam, dW, db, hist, it = O.fas_adjoint(W, b, U, lamN, h, m, 2, 1, relax, k, layer, TANH,
                                              init=2, Lam_init=Linit)
        lo = max(0, N - ((per_cycle * k + 1) * m - 1))    # exact from the top down to point lo
        assert np.abs(Lam[lo:] - Ls[lo:]).max() < 1e-12, k
        if (per_cycle * k + 1) * m <= N:
            assert np.abs(Lam[0] - Ls[0]).max() > 1e-8
    np.testing.assert_allclose(Lam, Ls, atol=1e-12)
    np.testing.assert_allclose(dW, dWs, atol=1e-12)
    np.testing.assert_allclose(db, dbs, atol=1e-12)


def test_adjoint_three_level_converges_to_serial_gradient():
    rng = np.random.default_rng(15)
    N, m = 32, 2
    W, b, u0 = _dense_problem(rng, N, 5, 3)
    U = O.serial_forward(W, b, u0, 1 / N, DENSE, TANH)
    lamN = rng.standard_normal(u0.shape)
    Ls, dWs, dbs = O.serial_backward(W, b, U, lamN, 1 / N, DENSE, TANH)
    Lam, dW, db, hist, it = O.fas_adjoint(W, b, U, lamN, 1 / N, m, 3, 1, O.RELAX_FCF, 30, DENSE, TANH,
                                          tol=1e-13)
    assert it < 30
    np.testing.assert_allclose(Lam, Ls, atol=1e-11)
    np.testing.assert_allclose(dW, dWs, atol=1e-11)


def test_adjoint_coarse_step_is_transpose_of_coarse_forward_jacobian():
    """<Psi_H(lam), v> == <lam, J v> with J the Jacobian of the coarse forward step (by differences)."""
    rng = np.random.default_rng(16)
    q, hs = 4, 0.6
    W, b, u0 = _dense_problem(rng, 1, q, 1)
    lam = rng.standard_normal((1, q))
    v = rng.standard_normal((1, q))
    eps = 1e-6
    Jv = (O.step(u0 + eps * v, W[0], b[0], hs, DENSE, TANH) - O.step(u0 - eps * v, W[0], b[0], hs, DENSE, TANH)) / (2 * eps)
    lhs = float(np.sum(O.adjoint_step(lam, u0, W[0], b[0], hs, DENSE, TANH) * v))
    assert abs(lhs - float(np.sum(lam * Jv))) < 1e-8


# ---------------------------------------------------------------------------------------
# Level maps against enumeration (integer work)
# ---------------------------------------------------------------------------------------
def test_level_map_vs_enumeration():
    for m in (2, 4, 8, 16):
        for N in list(range(1, 70)) + [256, 512, 1024, 4096]:
            for max_levels in (1, 2, 3, 5):
                for min_coarse in (1, 8):
                    # enumeration: level l holds every fine index divisible by m^l
                    # (a level with fewer than m steps has no whole coarse interval and is the coarsest)
                    sizes, fidx = O.level_map(N, m, max_levels, min_coarse)
                    for l in range(len(sizes)):
                        assert sizes[l] == len([n for n in range(1, N + 1) if n % (m ** l) == 0])
                        if l + 1 < len(sizes):
                            assert sizes[l] > min_coarse and sizes[l] >= m
                    last = sizes[-1]
                    assert len(sizes) == max_levels or last <= max(min_coarse, 1) or last < m
                    for l, idx in enumerate(fidx):
                        brute = [n for n in range(N + 1) if n % (m ** l) == 0]
                        assert list(idx) == brute


def test_named_hierarchies():
    assert O.level_sizes(16, 4, 2, 1) == [16, 4]
    assert O.level_sizes(256, 4, 3, 1) == [256, 64, 16]
    assert O.level_sizes(64, 4, 2, 1) == [64, 16]
    assert O.level_sizes(512, 8, 3, 1) == [512, 64, 8]
    assert O.level_sizes(1024, 16, 8, 8) == [1024, 64, 4]


# ---------------------------------------------------------------------------------------
# Depth-independent convergence (Sec. IV-A): recorded, with only a loose assertion
# ---------------------------------------------------------------------------------------
def test_convergence_history_similar_across_depths():
    its = []
    for N in (32, 64, 128):
        rng = np.random.default_rng(17)
        q = 8
        # weights smooth in depth (one matrix for all layers): the setting of an ODE discretisation
        A = rng.standard_normal((q, q)) / math.sqrt(q)
        W = np.tile(A, (N, 1, 1))
        b = np.zeros((N, q))
        u0 = rng.standard_normal((2, q))
        _, hist, it = O.fas_forward(W, b, u0, 1.0 / N, 4, 2, 1, O.RELAX_FCF, 20, DENSE, TANH, tol=1e-9)
        its.append(it)
    assert max(its) - min(its) <= 1, its


# ---------------------------------------------------------------------------------------
# Nested-iteration start (init = 3): coarse problems first, handed up level by level
# ---------------------------------------------------------------------------------------
def _euler_dense(v, Wn, bn, step_size, kind):
    z = v @ Wn.T + bn
    return v + step_size * (np.tanh(z) if kind == TANH else np.maximum(z, 0.0))


@pytest.mark.parametrize("kind", [TANH, RELU])
def test_nested_start_two_level_is_coarse_forward_euler(kind):
    """Two levels: the start values of the C-points are forward Euler with step c*h through every
    c-th layer's parameters (Sec. III-C, Eq. (25)), written out here without the oracle's helpers."""
    rng = np.random.default_rng(31)
    N, m, q = 12, 3, 5
    W, b, u0 = _dense_problem(rng, N, q, 2, scale=1.5)
    h = 0.4
    U, hist, it = O.fas_forward(W, b, u0, h, m, 2, 1, O.RELAX_F, 0, DENSE, kind, init=3)
    assert it == 0 and hist == []
    v = u0.copy()
    for i in range(1, N // m + 1):
        n = (i - 1) * m
        v = _euler_dense(v, W[n], b[n], m * h, kind)
        assert np.abs(U[i * m] - v).max() < 1e-14
    assert np.array_equal(U[0], u0)


def test_nested_start_three_level_brute_force():
    rng = np.random.default_rng(32)
    N, m, q = 16, 2, 4
    W, b, u0 = _dense_problem(rng, N, q, 3, scale=1.5)
    h = 0.3
    U, _, _ = O.fas_forward(W, b, u0, h, m, 3, 1, O.RELAX_FCF, 0, DENSE, TANH, init=3)
    # level 2: points at fine layers 0, 4, 8, 12, 16, step 4h
    lvl2 = [u0.copy()]
    for j in range(1, N // 4 + 1):
        n = (j - 1) * 4
        lvl2.append(_euler_dense(lvl2[-1], W[n], b[n], 4 * h, TANH))
    # level 1: points at fine layers 0, 2, .., 16, step 2h; even points from level 2, odd ones by one step
    for j2 in range(N // 4 + 1):
        assert np.abs(U[4 * j2] - lvl2[j2]).max() < 1e-14
    for j2 in range(N // 4):
        n = 4 * j2
        f_point = _euler_dense(lvl2[j2], W[n], b[n], 2 * h, TANH)
        assert np.abs(U[n + 2] - f_point).max() < 1e-14


def test_nested_start_three_level_brute_force_with_trailing_f_points():
    """N = 7, m = 2: levels of 7, 3 and 1 steps.  Level 2 holds fine layers 0 and 4; on level 1 point 2
    (fine layer 4) is injected, point 1 (layer 2) follows layer 0 and the trailing point 3 (layer 6)
    follows layer 4, each by one step of 2h."""
    rng = np.random.default_rng(33)
    N, m, q, h = 7, 2, 3, 0.3
    W, b, u0 = _dense_problem(rng, N, q, 2, scale=1.5)
    U, _, _ = O.fas_forward(W, b, u0, h, m, 3, 1, O.RELAX_FCF, 0, DENSE, TANH, init=3)
    u4 = _euler_dense(u0, W[0], b[0], 4 * h, TANH)
    u2 = _euler_dense(u0, W[0], b[0], 2 * h, TANH)
    u6 = _euler_dense(u4, W[4], b[4], 2 * h, TANH)
    for n, ref in ((0, u0), (2, u2), (4, u4), (6, u6)):
        assert np.abs(U[n] - ref).max() < 1e-14
    assert np.abs(U[1::2]).max() == 0.0               # fine F-points are left for the first relaxation


def test_nested_start_exact_for_layer_independent_constant_F():
    """W = 0 and the same bias in every layer: F is one constant, every step size integrates it
    exactly, so the start is already the solution and the first residual vanishes."""
    rng = np.random.default_rng(33)
    N, m, q = 32, 4, 3
    W = np.zeros((N, q, q))
    b = np.tile(rng.standard_normal((1, q)), (N, 1))
    u0 = rng.standard_normal((2, q))
    Us = O.serial_forward(W, b, u0, 0.1, DENSE, TANH)
    U, hist, _ = O.fas_forward(W, b, u0, 0.1, m, 3, 1, O.RELAX_F, 1, DENSE, TANH, init=3)
    assert hist[0] < 1e-13 and np.abs(U - Us).max() < 1e-13
    # the copy start is not exact here (guards against the test passing vacuously)
    _, hist_c, _ = O.fas_forward(W, b, u0, 0.1, m, 3, 1, O.RELAX_F, 1, DENSE, TANH, init=1)
    assert hist_c[0] > 1e-3


def test_nested_start_same_limit_and_smaller_first_residual():
    """Parameters that vary smoothly with depth (the regime of Sec. II, Eq. (2), where a coarse step
    approximates c fine ones): same limit as any other start, smaller residuals on the way."""
    rng = np.random.default_rng(34)
    N, m, q = 64, 4, 6
    Wa, Wb = rng.standard_normal((2, q, q)) / math.sqrt(q)
    t = np.arange(N) / N
    W = np.cos(2 * t)[:, None, None] * Wa + np.sin(2 * t)[:, None, None] * Wb
    b = np.outer(np.cos(t), rng.standard_normal(q)) * 0.3
    u0 = rng.standard_normal((3, q))
    h = 1 / N
    Us = O.serial_forward(W, b, u0, h, DENSE, TANH)
    U, hist, it = O.fas_forward(W, b, u0, h, m, 3, 1, O.RELAX_FCF, 30, DENSE, TANH, tol=1e-12, init=3)
    assert it < 30 and np.abs(U - Us).max() < 1e-10
    _, hist_c, it_c = O.fas_forward(W, b, u0, h, m, 3, 1, O.RELAX_FCF, 30, DENSE, TANH, tol=1e-12, init=1)
    assert hist[0] < 0.6 * hist_c[0] and hist[1] < 0.6 * hist_c[1] and it <= it_c


@pytest.mark.parametrize("layer", [DENSE, CONV])
def test_nested_start_same_limit_random_layers(layer):
    rng = np.random.default_rng(36)
    N, m = 32, 2
    if layer == DENSE:
        W, b, u0 = _dense_problem(rng, N, 6, 3)
    else:
        W, b, u0 = _conv_problem(rng, N, 2, 1, 4, 4)
    Us = O.serial_forward(W, b, u0, 1 / N, layer, TANH)
    U, hist, it = O.fas_forward(W, b, u0, 1 / N, m, 3, 1, O.RELAX_FCF, 30, layer, TANH, tol=1e-13, init=3)
    assert it < 30 and np.abs(U - Us).max() < 1e-11


def test_nested_start_adjoint_two_level_brute_force():
    """Adjoint solve: the start values of the C-points are the coarse adjoint recursion from the top,
    each coarse step using the state and parameters of the first layer of its interval."""
    rng = np.random.default_rng(35)
    N, m, q = 8, 4, 4
    W, b, u0 = _dense_problem(rng, N, q, 2, scale=1.5)
    h = 0.25
    Us = O.serial_forward(W, b, u0, h, DENSE, TANH)
    lamN = rng.standard_normal(u0.shape)
    Lam, dW, db, hist, it = O.fas_adjoint(W, b, Us, lamN, h, m, 2, 1, O.RELAX_F, 0, DENSE, TANH, init=3)
    lam = lamN.copy()
    assert np.array_equal(Lam[N], lamN)
    for i in range(N // m - 1, -1, -1):
        n = i * m
        z = Us[n] @ W[n].T + b[n]
        G = (1.0 - np.tanh(z) ** 2) * lam
        lam = lam + (m * h) * (G @ W[n])
        assert np.abs(Lam[n] - lam).max() < 1e-14


# ---------------------------------------------------------------------------------------
# Fully connected layers inside a convolution stack (Sec. IV-E): the kind itself, a mixed serial
# propagation and its gradient against the float64 library routines, and the multigrid limit
# ---------------------------------------------------------------------------------------
def _mixed_problem(rng, N, C, B, H, Wd, P):
    d = H * Wd * C
    Ws, bs, kinds = [], [], []
    for n in range(N):
        if n % P == 0:
            Ws.append(rng.standard_normal((d, d)) / math.sqrt(d)); bs.append(rng.standard_normal(d) * 0.3)
            kinds.append(O.FC)
        else:
            Ws.append(rng.standard_normal((C, 3, 3, C)) * math.sqrt(2.0 / (9 * C)))
            bs.append(rng.standard_normal(C) * 0.3); kinds.append(CONV)
    return Ws, bs, kinds, rng.standard_normal((B, H, Wd, C))


def _torch_mixed_forward(Ws, bs, kinds, x, h, f):
    for Wn, bn, kn in zip(Ws, bs, kinds):
        if kn == O.FC:
            z = torch.nn.functional.linear(x.reshape(x.shape[0], -1), Wn, bn).reshape(x.shape)
        else:
            z = torch.nn.functional.conv2d(x.permute(0, 3, 1, 2), Wn.permute(0, 3, 1, 2), bn,
                                           padding=1).permute(0, 2, 3, 1)
        x = x + h * f(z)
    return x


@pytest.mark.parametrize("kind", [TANH, RELU])
def test_fully_connected_step_on_an_image_state_matches_torch_linear(kind):
    rng = np.random.default_rng(41)
    Ws, bs, kinds, u0 = _mixed_problem(rng, 1, 3, 2, 4, 5, 1)
    got = O.step(u0, Ws[0], bs[0], 0.3, O.FC, kind)
    f = torch.tanh if kind == TANH else torch.relu
    ref = _torch_mixed_forward([torch.from_numpy(Ws[0])], [torch.from_numpy(bs[0])], kinds, torch.from_numpy(u0), 0.3, f)
    np.testing.assert_allclose(got, ref.numpy(), rtol=1e-13, atol=1e-13)
    # flattening order is the storage order of the sample: row y, column x, channel c
    e = np.zeros_like(u0); e[1, 2, 3, 1] = 1.0
    z = O.affine(e, Ws[0], np.zeros_like(bs[0]), O.FC)
    np.testing.assert_allclose(z[1].reshape(-1), Ws[0][:, (2 * 5 + 3) * 3 + 1], rtol=0, atol=0)
    assert not z[0].any()


def test_mixed_stack_serial_forward_and_gradient_vs_autograd():
    rng = np.random.default_rng(42)
    N, h, P = 7, 1.0 / 7, 3
    Ws, bs, kinds, u0 = _mixed_problem(rng, N, 2, 2, 3, 4, P)
    assert kinds == [O.FC, CONV, CONV, O.FC, CONV, CONV, O.FC]
    Cw = rng.standard_normal(u0.shape)
    U = O.serial_forward(Ws, bs, u0, h, kinds, TANH)
    Lam, dW, db = O.serial_backward(Ws, bs, U, Cw, h, kinds, TANH)
    Wt = [torch.tensor(w, requires_grad=True) for w in Ws]
    bt = [torch.tensor(b, requires_grad=True) for b in bs]
    ut = torch.tensor(u0, requires_grad=True)
    x = _torch_mixed_forward(Wt, bt, kinds, ut, h, torch.tanh)
    np.testing.assert_allclose(U[-1], x.detach().numpy(), rtol=1e-12, atol=1e-13)
    (x * torch.tensor(Cw)).sum().backward()
    for n in range(N):
        np.testing.assert_allclose(dW[n], Wt[n].grad.numpy(), rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(db[n], bt[n].grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(Lam[0], ut.grad.numpy(), rtol=1e-10, atol=1e-13)
    dW2, db2 = O.parameter_gradient(Ws, bs, U, Lam, h, kinds, TANH)
    for n in range(N):
        np.testing.assert_allclose(dW2[n], dW[n], rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("P", [4, 3, 16])
def test_mixed_stack_two_level_exactness_forward_and_adjoint(P):
    """The fully connected layers sit on C-points (P = 4), on F-points too (P = 3), or only at layer 0."""
    rng = np.random.default_rng(43)
    N, m, h = 12, 4, 1.0 / 12
    Ws, bs, kinds, u0 = _mixed_problem(rng, N, 2, 2, 3, 3, P)
    Us = O.serial_forward(Ws, bs, u0, h, kinds, TANH)
    U, hist, it = O.fas_forward(Ws, bs, u0, h, m, 2, 1, O.RELAX_F, N // m, kinds, TANH)
    assert np.abs(U - Us).max() < 1e-12 and hist[-1] < hist[0]
    U1, _, _ = O.fas_forward(Ws, bs, u0, h, m, 2, 1, O.RELAX_F, 1, kinds, TANH)
    assert np.abs(U1[:m + 1] - Us[:m + 1]).max() < 1e-12 and np.abs(U1[-1] - Us[-1]).max() > 1e-6
    lamN = rng.standard_normal(u0.shape)
    Ls, dWs, dbs = O.serial_backward(Ws, bs, Us, lamN, h, kinds, TANH)
    Lam, dW, db, _, _ = O.fas_adjoint(Ws, bs, Us, lamN, h, m, 2, 1, O.RELAX_F, N // m, kinds, TANH)
    assert np.abs(Lam - Ls).max() < 1e-12
    for n in range(N):
        assert np.abs(dW[n] - dWs[n]).max() < 1e-12 and np.abs(db[n] - dbs[n]).max() < 1e-12
    r = O.residual_norm(Ws, bs, u0, Us, h, kinds, TANH)
    assert r < 1e-12 and O.residual_norm(Ws, bs, u0, U1, h, kinds, TANH) > 1e-6


# ---------------------------------------------------------------------------------------
# Stored reference of the smallest benchmark workload (written by tests/golden/make_cfg1_oracle.py)
# ---------------------------------------------------------------------------------------
def test_stored_cfg1_reference_is_what_the_oracle_computes_today():
    import importlib.util
    import json
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_cfg1_oracle", os.path.join(here, "make_cfg1_oracle.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    with open(os.path.join(here, "cfg1_oracle.json")) as f:
        stored = json.load(f)
    assert stored["cycles"] == now["cycles"] == 4
    for key in ("U", "Lam", "dW", "db", "residual_history", "adjoint_residual_history"):
        a, b = np.asarray(stored[key]), np.asarray(now[key])
        assert a.shape == b.shape and np.abs(a - b).max() <= 1e-13 * max(1.0, np.abs(b).max()), key
    # and the stored iterate is the exact solution: N/m = 4 cycles of two-level F-relaxation
    import mgrit_inputs as I
    wl = I.cfg1()
    d = I.generate(wl)
    Us = O.serial_forward(d["W"], d["b"], d["u0"], wl.h, wl.layer, wl.act)
    assert np.abs(np.asarray(stored["U"]) - Us).max() < 1e-12
