"""Seeded random small workloads through the C-ABI library against the oracle: layer kind, activation, operand
type, depth, coarsening factor, level count, relaxation, initial guess, batch and width / channels / image size are
drawn at random (fixed seed), so that index maps, ragged tiles and trailing F-points meet in combinations the
hand-picked cases do not list.  Forward solve, then adjoint solve and parameter gradient about the oracle's states.
"""
import numpy as np
import pytest

import mgrit_inputs as I
from oracle import mgrit_oracle as O
from tests.gpu_util import GpuProblem, oracle_forward, oracle_adjoint, rel_l2_per_state

pytestmark = pytest.mark.gpu
TOL = {I.FP32: 1e-5, I.BF16: 2e-2}


def _draw(rng, idx):
    dense = bool(rng.integers(0, 2))
    dtype = I.BF16 if rng.integers(0, 3) == 0 else I.FP32
    act = I.TANH if rng.integers(0, 2) else I.RELU
    m = int(rng.integers(2, 6))
    N = int(rng.integers(m, 41))
    kw = dict(N=N, m=m, max_levels=int(rng.integers(2, 4)), min_coarse=int(rng.integers(1, 4)),
              relax=int(rng.integers(0, 2)), max_iter=int(rng.integers(1, 4)), act=act, dtype=dtype, head_classes=0,
              bias_var=0.1, seed=1000 + idx)
    if dense:
        kw.update(q=8 * int(rng.integers(1, 26)), B=int(rng.integers(1, 70)))
        base = I.cfg5(1)
        name = f"rand{idx}_dense_q{kw['q']}_B{kw['B']}"
    else:
        kw.update(C=int(rng.choice([8, 16, 24, 32, 48, 64])), Himg=int(rng.integers(1, 13)), Wimg=int(rng.integers(1, 13)),
                  B=int(rng.integers(1, 5)), lifted_input=False)
        base = I.cfg4(1)
        name = f"rand{idx}_conv_c{kw['C']}_{kw['Himg']}x{kw['Wimg']}_B{kw['B']}"
    name += f"_N{N}_m{m}_L{kw['max_levels']}_{'FCF' if kw['relax'] else 'F'}_{'bf16' if dtype else 'fp32'}_{'relu' if act else 'tanh'}"
    return I.reduced(base, name=name, **kw), int(rng.choice([0, 1, 3]))


_RNG = np.random.default_rng(20260707)
CASES = [_draw(_RNG, i) for i in range(64)]


@pytest.mark.parametrize("wl,init", CASES, ids=lambda v: v.name if hasattr(v, "name") else f"init{v}")
def test_random_workload_forward_and_adjoint(wl, init):
    print(f"\n[case] {wl.name} init={init} cycles={wl.max_iter}", flush=True)
    data = I.generate(wl)
    gp = GpuProblem(wl, data, init=init)
    sizes, fine = gp.M.mgrit_level_map(gp.p)
    sizes_o, fine_o = O.level_map(wl.N, wl.m, wl.max_levels, wl.min_coarse)
    assert sizes == sizes_o and all(list(a) == list(b) for a, b in zip(fine, fine_o))     # integer maps: bit-exact
    _, U, hist, it = gp.forward()
    Uo, hist_o, it_o = oracle_forward(wl, data, init=init)
    tol = TOL[wl.dtype]
    assert it == it_o
    assert rel_l2_per_state(U, Uo) <= tol, rel_l2_per_state(U, Uo)
    # a residual that the oracle sees converge to 1e-16 stops at the float32 rounding floor on the GPU: one ulp of
    # the largest state value per summed entry
    floor = 2.0 ** -23 * float(np.abs(Uo).max()) * np.sqrt((sizes[1] + 1) * wl.E if len(sizes) > 1 else 1.0)
    for a, b in zip(hist, hist_o):
        assert abs(a - b) <= (1e-3 if wl.dtype == I.FP32 else 0.2) * abs(b) + floor, (hist, hist_o, floor)
    # ReLU' is a 0/1 decision on the sign of z that float32 summation order can flip (one flip moves a gradient
    # entry by O(1), far above 1e-5), so the float + ReLU cases stop after the forward solve; bf16 cases linearise
    # about bf16-representable states, so that both sides take the decisions from the same operand values
    if wl.dtype == I.FP32 and wl.act == I.RELU:
        return
    Ulin = Uo.astype(np.float32) if wl.dtype == I.FP32 else I.round_to_bf16(Uo.astype(np.float32))
    lamN = np.random.default_rng(wl.seed + 7).standard_normal(wl.state_shape).astype(np.float32)
    gpa = GpuProblem(wl, data, init=init)
    Lam, dW, db, hist_a, it_a = gpa.adjoint(Ulin, lamN)
    Lo, dWo, dbo, hist_ao, it_ao = oracle_adjoint(wl, data, Ulin, lamN, init=init)
    eL, eW, eb = rel_l2_per_state(Lam, Lo), rel_l2_per_state(dW, dWo), rel_l2_per_state(db, dbo)
    print(f"{wl.name}: Lam {eL:.2e} dW {eW:.2e} db {eb:.2e}", flush=True)
    assert it_a == it_ao
    assert eL <= tol and eW <= tol and eb <= tol, (eL, eW, eb)
