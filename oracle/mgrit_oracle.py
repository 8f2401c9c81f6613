"""CPU oracle for the layer-parallel multigrid (MGRIT-FAS) solve of a residual network.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP path is
checked against.  It shares no code with the HIP path and must never be imported by the
product package; only tests, the smoke check and the benchmark's CPU-baseline leg use it.

Everything is float64 numpy.  A matrix product (`@`) is the only library primitive used as
a step; there is no blocking, fusion or reordering beyond what the formulas state.

What is computed, and where the paper defines it
------------------------------------------------
* layer step  Phi(u) = u + h F(u; theta),  F = activation(affine map + bias)   [Sec. II, Eq. (1)]
* serial forward propagation over n = 0..N-1                                   [Sec. II, Eq. (1)]
* the fine-level system L_h(U) = f_h and its residual R_h = f_h - L_h(U)      [Sec. III-C, Eq. (18)-(19)]
* coarse levels by injection of every c-th layer (state, residual, parameters),
  coarse operator with step H = c h                                            [Sec. III-C, Eq. (23)-(25)]
* F-/C-/FCF-relaxation                                                         [Sec. III-C, Fig. 3]
* the FAS right-hand side S_H and the coarse-to-fine update                    [Sec. III-B, Eq. (14)-(17)]
* the two-level FAS scheme, applied recursively as a V-cycle                   [Sec. III-A; Sec. III-C, Alg. 1]
* the adjoint (backward) solve: the paper states that the same multigrid removes the
  serial backward propagation but prints no equations; here it is the exact reverse-mode
  derivative of Eq. (1), solved by the same cycle on the reversed layer axis.
* the nested-iteration start (init = 3): the paper prints no start-up procedure; the coarsest
  level's equation is solved first and handed up level by level                [Sec. III-A background]
* stacks that mix layer kinds (blocks of one fully connected layer followed by convolution
  layers): `layer` may be a sequence with one kind per layer, W and b then are sequences of
  per-layer arrays; the fully connected kind FC acts on the flattened sample   [Sec. IV-E]

Index convention: N layer steps, N+1 states u^0..u^N, parameters theta^0..theta^{N-1}.
Level l has N_l = N / c^l steps and step size h_l = c^l h; level-l point j is fine layer
j c^l and uses theta^{j c^l}.  (The paper writes the coarsening factor as c; the public
interface of this project calls it m.)

Pins (tests/test_oracle_pins.py): two-level exactness after N/c cycles, fixed point at the
serial solution, linear-F closed forms and the dense two-grid and three-grid operators, brute-force coarse
equation check, layer steps against an independent float64 library routine, gradients
against finite differences and automatic differentiation, level maps against enumeration;
the nested-iteration start against hand-written coarse forward-Euler loops, its exactness for a
layer-independent constant F, and the unchanged fixed point; the fully connected kind and mixed
stacks against the float64 library routines, automatic differentiation and two-level exactness.
A multilevel (3+ level) iterate at a fixed finite cycle count is pinned for linear F by the dense
three-grid correction scheme (relax, restrict, one two-grid cycle on the middle level, correct);
for nonlinear F it rests on that pin of the recursion together with the two-level pins of the
nonlinear pieces, its limit and its fixed point -- no independent value of a nonlinear
three-level iterate exists to compare with.
"""
from __future__ import annotations

import numpy as np

DENSE, CONV, FC = 0, 1, 2          # FC: fully connected on the flattened sample of an image state
TANH, RELU, IDENT = 0, 1, 2
RELAX_F, RELAX_FCF = 0, 1


# ----------------------------------------------------------------------------------------
# Layer step, Eq. (1)
# ----------------------------------------------------------------------------------------
def act(z, kind):
    if kind == TANH:
        return np.tanh(z)
    if kind == RELU:
        return np.maximum(z, 0.0)
    return z


def act_prime(z, kind):
    """Derivative of the activation at the pre-activation z; ReLU'(0) = 0."""
    if kind == TANH:
        return 1.0 - np.tanh(z) ** 2
    if kind == RELU:
        return (z > 0.0).astype(np.float64)
    return np.ones_like(z)


def affine(u, Wn, bn, layer):
    """Pre-activation z = A u + b.

    dense: u [B,q], Wn [q_out,q_in]:  z[r,o] = sum_i Wn[o,i] u[r,i] + bn[o]
    conv:  u [B,H,W,C] (NHWC), Wn [C_out,3,3,C_in], stride 1, zero padding of one pixel,
           cross-correlation: z[b,y,x,o] = sum_{dy,dx,i} Wn[o,dy,dx,i] u[b,y+dy-1,x+dx-1,i] + bn[o]
    """
    if layer == DENSE:
        return u @ Wn.T + bn
    if layer == FC:                       # u [B,...] flattened per sample to [B,d]; Wn [d,d], bn [d]
        return (u.reshape(u.shape[0], -1) @ Wn.T + bn).reshape(u.shape)
    B, H, W, C = u.shape
    up = np.zeros((B, H + 2, W + 2, C))
    up[:, 1:-1, 1:-1, :] = u
    z = np.zeros((B, H, W, Wn.shape[0]))
    for dy in range(3):
        for dx in range(3):
            z += up[:, dy:dy + H, dx:dx + W, :] @ Wn[:, dy, dx, :].T
    return z + bn


def affine_T(G, Wn, layer):
    """Transpose of the linear part of `affine`: returns A^T G (same shape as the state)."""
    if layer == DENSE:
        return G @ Wn
    if layer == FC:
        return (G.reshape(G.shape[0], -1) @ Wn).reshape(G.shape)
    B, H, W, _ = G.shape
    C = Wn.shape[3]
    gp = np.zeros((B, H + 2, W + 2, C))
    for dy in range(3):
        for dx in range(3):
            gp[:, dy:dy + H, dx:dx + W, :] += G @ Wn[:, dy, dx, :]
    return gp[:, 1:-1, 1:-1, :]


def weight_grad(G, u, layer):
    """Gradient of sum(G * affine(u)) with respect to (Wn, bn)."""
    if layer == DENSE:
        return G.T @ u, G.sum(axis=0)
    if layer == FC:
        G2, u2 = G.reshape(G.shape[0], -1), u.reshape(u.shape[0], -1)
        return G2.T @ u2, G2.sum(axis=0)
    B, H, W, C = u.shape
    Co = G.shape[3]
    up = np.zeros((B, H + 2, W + 2, C))
    up[:, 1:-1, 1:-1, :] = u
    dK = np.zeros((Co, 3, 3, C))
    G2 = G.reshape(-1, Co)
    for dy in range(3):
        for dx in range(3):
            dK[:, dy, dx, :] = G2.T @ up[:, dy:dy + H, dx:dx + W, :].reshape(-1, C)
    return dK, G2.sum(axis=0)


def _f64(x):
    """float64 copy of an array, or of every array of a per-layer sequence (mixed stacks)."""
    if isinstance(x, (list, tuple)):
        return [np.asarray(v, np.float64) for v in x]
    return np.asarray(x, np.float64)


def _zeros_like(x):
    return [np.zeros_like(v) for v in x] if isinstance(x, list) else np.zeros_like(x)


def _kind_of(layer, n):
    """Kind of layer n: `layer` is one kind for the whole stack or a sequence of per-layer kinds."""
    return layer[n] if isinstance(layer, (list, tuple, np.ndarray)) else layer


def step(u, Wn, bn, hs, layer, kind):
    """Phi(u) = u + hs * F(u; theta), Eq. (1) with step size hs."""
    return u + hs * act(affine(u, Wn, bn, layer), kind)


def adjoint_step(lam, u_lin, Wn, bn, hs, layer, kind):
    """Psi(lam) = lam + hs * (dF/du at u_lin)^T lam  -- transpose of the Jacobian of `step`."""
    G = act_prime(affine(u_lin, Wn, bn, layer), kind) * lam
    return lam + hs * affine_T(G, Wn, layer)


# ----------------------------------------------------------------------------------------
# Serial propagation (the plain definition the multigrid iteration converges to)
# ----------------------------------------------------------------------------------------
def serial_forward(W, b, u0, h, layer, kind):
    W = _f64(W)
    b = _f64(b)
    N = len(W)
    U = np.zeros((N + 1,) + u0.shape)
    U[0] = u0
    for n in range(N):
        U[n + 1] = step(U[n], W[n], b[n], h, _kind_of(layer, n), kind)
    return U


def serial_backward(W, b, U, lamN, h, layer, kind):
    """Reverse-mode derivative of serial propagation, linearised about the given states U.

    z^n = A_n U^n + b_n; G^n = act'(z^n) * lam^{n+1}; lam^n = lam^{n+1} + h A_n^T G^n;
    dA_n = h G^n (U^n)^T summed over the batch; db_n = h sum G^n.
    """
    W = _f64(W)
    b = _f64(b)
    U = np.asarray(U, np.float64)
    N = len(W)
    Lam = np.zeros_like(U)
    Lam[N] = lamN
    dW = _zeros_like(W)
    db = _zeros_like(b)
    for n in range(N - 1, -1, -1):
        ln = _kind_of(layer, n)
        G = act_prime(affine(U[n], W[n], b[n], ln), kind) * Lam[n + 1]
        Lam[n] = Lam[n + 1] + h * affine_T(G, W[n], ln)
        gW, gb = weight_grad(G, U[n], ln)
        dW[n] = h * gW
        db[n] = h * gb
    return Lam, dW, db


def parameter_gradient(W, b, U, Lam, h, layer, kind):
    """dtheta from given (possibly approximate) states U and adjoints Lam, layer by layer."""
    W = _f64(W)
    b = _f64(b)
    N = len(W)
    dW = _zeros_like(W)
    db = _zeros_like(b)
    for n in range(N):
        ln = _kind_of(layer, n)
        G = act_prime(affine(U[n], W[n], b[n], ln), kind) * Lam[n + 1]
        gW, gb = weight_grad(G, U[n], ln)
        dW[n] = h * gW
        db[n] = h * gb
    return dW, db


# ----------------------------------------------------------------------------------------
# Level hierarchy: every c-th layer of a level also belongs to the next coarser level
# ----------------------------------------------------------------------------------------
def level_sizes(N, m, max_levels, min_coarse):
    """Number of steps on each level.  Coarsening continues while fewer than max_levels levels
    exist and the current level has more than min_coarse steps and at least one whole coarse
    interval (m steps).  The C-points of a level are its points 0, m, 2m, ...; a level whose size
    is not a multiple of m ends in fewer than m trailing F-points behind its last C-point (the
    paper does not treat this case; every m-th layer is coarse, Sec. III-C, so the rest can only
    be fine), and the next level has floor(N_l / m) steps."""
    if N < 1 or m < 2 or max_levels < 1:
        raise ValueError("invalid hierarchy parameters")
    sizes = [N]
    while len(sizes) < max_levels and sizes[-1] > max(min_coarse, 1) and sizes[-1] >= m:
        sizes.append(sizes[-1] // m)
    return sizes


def level_map(N, m, max_levels, min_coarse):
    """(sizes, fine_index): fine_index[l][j] = fine layer index of point j on level l."""
    sizes = level_sizes(N, m, max_levels, min_coarse)
    fine_index = [np.arange(Nl + 1, dtype=np.int64) * (m ** l) for l, Nl in enumerate(sizes)]
    return sizes, fine_index


# ----------------------------------------------------------------------------------------
# The FAS cycle, Alg. 1, written for a generic propagator so that the forward and the adjoint
# solve are the same code.  phi(l, j, u) maps the state at point j of level l to point j+1.
# ----------------------------------------------------------------------------------------
def _f_relax(l, U, g, m, phi):
    Nl = U.shape[0] - 1
    n_int = Nl // m
    for i in range(n_int):
        for k in range(1, m):
            j = i * m + k
            U[j] = phi(l, j - 1, U[j - 1]) + g[j]
    for j in range(n_int * m + 1, Nl + 1):         # trailing F-points behind the last C-point
        U[j] = phi(l, j - 1, U[j - 1]) + g[j]


def _c_relax(l, U, g, m, phi):
    n_int = (U.shape[0] - 1) // m
    for i in range(1, n_int + 1):
        j = i * m
        U[j] = phi(l, j - 1, U[j - 1]) + g[j]


def _cycle(l, sizes, U, g, m, relax, phi, hist):
    L = len(sizes)
    Nl = sizes[l]
    if l == L - 1:                                   # coarsest level: solve exactly, in sequence
        U[0] = g[0]
        for j in range(1, Nl + 1):
            U[j] = phi(l, j - 1, U[j - 1]) + g[j]
        return
    Nc = sizes[l + 1]
    # step 1: relaxation
    _f_relax(l, U, g, m, phi)
    if relax == RELAX_FCF:
        _c_relax(l, U, g, m, phi)
        _f_relax(l, U, g, m, phi)
    # residual R = f - L(U) at the C-points
    r = np.zeros((Nc + 1,) + U.shape[1:])
    r[0] = g[0] - U[0]
    for i in range(1, Nc + 1):
        r[i] = g[i * m] - U[i * m] + phi(l, i * m - 1, U[i * m - 1])
    if l == 0 and hist is not None:
        hist.append(float(np.sqrt(np.sum(r * r))))
    # step 2: restriction by injection
    Ubar = U[::m].copy()
    # step 3: right-hand side S_H = L_H(Ubar) + R_H, then solve L_H(V) = S_H
    gH = np.zeros_like(Ubar)
    gH[0] = Ubar[0] + r[0]
    for i in range(1, Nc + 1):
        gH[i] = Ubar[i] - phi(l + 1, i - 1, Ubar[i - 1]) + r[i]
    V = Ubar.copy()
    _cycle(l + 1, sizes, V, gH, m, relax, phi, None)
    # steps 4, 5: coarse error and C-point update
    for i in range(Nc + 1):
        U[i * m] += V[i] - Ubar[i]
    # F-points follow the corrected C-points
    _f_relax(l, U, g, m, phi)


def _nested_start(sizes, m, phi, first, shape):
    """Nested-iteration start (the paper's multigrid background, Sec. III-A, solves coarse problems
    first; the paper prints no start-up procedure for Alg. 1, so this is the plain one): every level
    carries the equation L(V) = (first, 0, .., 0) with its own step size.  The coarsest level is
    solved in sequence; going up, the C-points of a level take the values of the next coarser level
    (injection the other way round) and its F-points follow by F-relaxation.  Returns the values of
    the points of level 1, i.e. the start values of the fine C-points."""
    L = len(sizes)
    V = np.zeros((sizes[L - 1] + 1,) + shape)
    V[0] = first
    for j in range(1, sizes[L - 1] + 1):
        V[j] = phi(L - 1, j - 1, V[j - 1])
    for l in range(L - 2, 0, -1):
        Ul = np.zeros((sizes[l] + 1,) + shape)
        Ul[::m] = V
        _f_relax(l, Ul, np.zeros_like(Ul), m, phi)
        V = Ul
    return V


def _solve(sizes, m, relax, phi, first, shape, init, X_init, max_iter, tol, norm_kind):
    N = sizes[0]
    L = len(sizes)
    U = np.zeros((N + 1,) + shape)
    if init == 1:
        U[::m] = first
    elif init == 2:
        U[:] = X_init
    elif init == 3 and L > 1:
        U[::m] = _nested_start(sizes, m, phi, first, shape)
    U[0] = first
    g = np.zeros_like(U)
    g[0] = first
    hist = []
    if L == 1:
        _cycle(0, sizes, U, g, m, relax, phi, None)
        return U, [0.0], 1
    count = (sizes[1] + 1) * int(np.prod(shape))
    iters = 0
    for _ in range(max_iter):
        _cycle(0, sizes, U, g, m, relax, phi, hist)
        if norm_kind == 1:
            hist[-1] /= np.sqrt(count)
        iters += 1
        if tol > 0 and hist[-1] <= tol:
            break
    return U, hist, iters


def fas_forward(W, b, u0, h, m, max_levels, min_coarse, relax, max_iter, layer, kind,
                tol=0.0, norm_kind=0, init=1, U_init=None):
    """Forward MGRIT-FAS solve.  Returns (U [N+1,...], residual history, cycles done)."""
    W = _f64(W)
    b = _f64(b)
    u0 = np.asarray(u0, np.float64)
    N = len(W)
    sizes = level_sizes(N, m, max_levels, min_coarse)

    def phi(l, j, u):
        n = j * m ** l
        return step(u, W[n], b[n], h * m ** l, _kind_of(layer, n), kind)

    return _solve(sizes, m, relax, phi, u0, u0.shape, init, U_init, max_iter, tol, norm_kind)


def fas_adjoint(W, b, U, lamN, h, m, max_levels, min_coarse, relax, max_iter, layer, kind,
                tol=0.0, norm_kind=0, init=1, Lam_init=None):
    """Adjoint MGRIT-FAS solve linearised about the states U, then the parameter gradient.

    The same cycle runs on the reversed layer axis, whose level-l point j' is fine point
    N - j' c^l: the sweep j' -> j'+1 is the adjoint step from fine point n + c^l to fine point
    n = N - (j'+1) c^l, which uses the state and parameters of fine layer n (the first layer of
    the coarse interval) and step h_l.
    Returns (Lam [N+1,...], dW, db, residual history, cycles done).
    """
    W = _f64(W)
    b = _f64(b)
    U = np.asarray(U, np.float64)
    lamN = np.asarray(lamN, np.float64)
    N = len(W)
    sizes = level_sizes(N, m, max_levels, min_coarse)

    def psi(l, jr, lam):
        n = N - (jr + 1) * m ** l          # reversed sweep jr -> jr+1 lands on fine point n (the hierarchy of
        #                                    the reversed axis counts from point N: its level-l point j is N - j c^l)
        return adjoint_step(lam, U[n], W[n], b[n], h * m ** l, _kind_of(layer, n), kind)

    Xi = None if Lam_init is None else np.asarray(Lam_init, np.float64)[::-1]
    LamR, hist, iters = _solve(sizes, m, relax, psi, lamN, lamN.shape, init, Xi, max_iter, tol,
                               norm_kind)
    Lam = LamR[::-1].copy()
    dW, db = parameter_gradient(W, b, U, Lam, h, layer, kind)
    return Lam, dW, db, hist, iters


def residual_norm(W, b, u0, U, h, layer, kind, norm_kind=0):
    """|| f_h - L_h(U) || over all N+1 points, Eq. (18)-(19)."""
    W = _f64(W)
    b = _f64(b)
    U = np.asarray(U, np.float64)
    N = len(W)
    s = float(np.sum((np.asarray(u0, np.float64) - U[0]) ** 2))
    for n in range(1, N + 1):
        r = step(U[n - 1], W[n - 1], b[n - 1], h, _kind_of(layer, n - 1), kind) - U[n]
        s += float(np.sum(r * r))
    nrm = np.sqrt(s)
    if norm_kind == 1:
        nrm /= np.sqrt(U.size)
    return nrm
