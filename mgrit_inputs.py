"""Seeded synthetic inputs for the layer-parallel multigrid (MGRIT-FAS) path.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic.  Both the CPU oracle's tests and the HIP path's tests and
benchmark take their inputs from here, so the two sides see identical arrays.

Recipe (one `numpy.random.default_rng(seed)` stream per workload, draw order
`W, b, u0 | y, K_in, W_o, labels`; everything drawn in float64 and cast to
float32; where the workload stores weights in bf16 the float32 weights are then
rounded to the nearest bf16 value, ties to even, and kept as float32 numbers that
are exactly representable in bf16):

  dense:  W[n] ~ N(0, 1/q) (variance), b[n] ~ N(0, bias_var) or 0, u0 ~ N(0, 1)
  conv:   K[n] ~ N(0, 2/(9 C)) (variance), b[n] ~ N(0, bias_var), NHWC states;
          u0 either ~N(0,1) directly or a one-channel image y ~ U[0,1] lifted to C
          channels by a fixed random 3x3 kernel K_in ~ N(0, 2/9) (the lifting is a
          plain data-preparation step done here with explicit shifts).
  mixed:  a conv workload with fc_period = P > 0: layers 0, P, 2P, ... are fully connected on the
          flattened sample (d = Himg Wimg C); Wfc[k] ~ N(0, 1/d), bfc[k] ~ N(0, bias_var), drawn after
          everything else, so the other arrays are those of the same workload without them.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

DENSE, CONV, FC = 0, 1, 2           # FC: a fully connected layer inside a conv stack (mixed workloads)
TANH, RELU = 0, 1
FP32, BF16 = 0, 1
RELAX_F, RELAX_FCF = 0, 1


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape and algorithm parameters of one synthetic MGRIT-FAS problem."""

    name: str
    layer: int                 # DENSE or CONV
    act: int                   # TANH or RELU
    dtype: int                 # FP32 or BF16 (weight storage / MFMA operand type)
    N: int                     # number of layer steps; states are u^0 .. u^N
    m: int                     # coarsening factor (the paper's c)
    max_levels: int
    relax: int                 # RELAX_F or RELAX_FCF
    max_iter: int
    B: int
    q: int = 0                 # dense width
    C: int = 0                 # conv channels
    Himg: int = 0
    Wimg: int = 0
    min_coarse: int = 1
    bias_var: float = 0.1      # 0 -> biases identically zero
    lifted_input: bool = False  # conv: u0 = fixed random 3x3 lift of a 1-channel U[0,1] image
    head_classes: int = 0      # >0: also draw a softmax head W_o and integer labels
    seed: int = 0
    tol: float = 0.0
    norm_kind: int = 0
    fc_period: int = 0          # conv only, > 0: every fc_period-th layer is fully connected on the flattened sample
    smooth_depth: bool = False  # True: parameters vary smoothly with depth (a quarter turn between two
                                # random draws) instead of being independent from layer to layer

    @property
    def h(self) -> float:
        return 1.0 / self.N

    @property
    def state_shape(self):
        if self.layer == DENSE:
            return (self.B, self.q)
        return (self.B, self.Himg, self.Wimg, self.C)

    @property
    def E(self) -> int:
        return int(np.prod(self.state_shape))

    @property
    def n_fc(self) -> int:
        return (self.N + self.fc_period - 1) // self.fc_period if self.fc_period else 0

    @property
    def d_fc(self) -> int:
        return self.Himg * self.Wimg * self.C


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(x.shape)


def _lift(y: np.ndarray, K_in: np.ndarray) -> np.ndarray:
    """u0[b,y,x,c] = sum_{dy,dx} K_in[c,dy,dx] * y_pad[b,y+dy,x+dx] (zero padding, no bias)."""
    B, H, W = y.shape
    yp = np.zeros((B, H + 2, W + 2), dtype=np.float64)
    yp[:, 1:-1, 1:-1] = y
    out = np.zeros((B, H, W, K_in.shape[0]), dtype=np.float64)
    for dy in range(3):
        for dx in range(3):
            out += yp[:, dy:dy + H, dx:dx + W, None] * K_in[None, None, None, :, dy, dx]
    return out


def generate(wl: Workload) -> dict:
    """Draw the arrays of a workload.  Returns float32 arrays (labels int64)."""
    rng = np.random.default_rng(wl.seed)
    out = {}
    if wl.layer == DENSE:
        W = rng.standard_normal((wl.N, wl.q, wl.q)) * np.sqrt(1.0 / wl.q)
        b = rng.standard_normal((wl.N, wl.q)) * np.sqrt(wl.bias_var) if wl.bias_var > 0 \
            else np.zeros((wl.N, wl.q))
        u0 = rng.standard_normal((wl.B, wl.q))
        feat = wl.q
    else:
        W = rng.standard_normal((wl.N, wl.C, 3, 3, wl.C)) * np.sqrt(2.0 / (9.0 * wl.C))
        b = rng.standard_normal((wl.N, wl.C)) * np.sqrt(wl.bias_var) if wl.bias_var > 0 \
            else np.zeros((wl.N, wl.C))
        if wl.lifted_input:
            y = rng.uniform(0.0, 1.0, (wl.B, wl.Himg, wl.Wimg))
            K_in = rng.standard_normal((wl.C, 3, 3)) * np.sqrt(2.0 / 9.0)
            u0 = _lift(y, K_in)
        else:
            u0 = rng.standard_normal((wl.B, wl.Himg, wl.Wimg, wl.C))
        feat = wl.C * wl.Himg * wl.Wimg
    if wl.smooth_depth:
        # theta(t) = cos(pi t / 2) theta_a + sin(pi t / 2) theta_b, t = n / N: same variance at every depth
        t = (np.arange(wl.N) / wl.N) * (np.pi / 2)
        ex = (slice(None),) + (None,) * (W.ndim - 1)
        W = np.cos(t)[ex] * W[0] + np.sin(t)[ex] * W[wl.N // 2]
        b = np.cos(t)[:, None] * b[0] + np.sin(t)[:, None] * b[wl.N // 2]
    W = W.astype(np.float32)
    if wl.dtype == BF16:
        W = round_to_bf16(W)
    out["W"] = W
    out["b"] = b.astype(np.float32)
    out["u0"] = np.ascontiguousarray(u0.astype(np.float32))
    if wl.head_classes > 0:
        out["W_o"] = (rng.standard_normal((wl.head_classes, feat)) * np.sqrt(1.0 / feat)).astype(np.float32)
        out["labels"] = rng.integers(0, wl.head_classes, size=(wl.B,))
    if wl.fc_period > 0:
        d = wl.d_fc
        Wfc = (rng.standard_normal((wl.n_fc, d, d)) * np.sqrt(1.0 / d)).astype(np.float32)
        out["Wfc"] = round_to_bf16(Wfc) if wl.dtype == BF16 else Wfc
        bfc = rng.standard_normal((wl.n_fc, d)) * np.sqrt(wl.bias_var) if wl.bias_var > 0 else np.zeros((wl.n_fc, d))
        out["bfc"] = bfc.astype(np.float32)
    return out


def per_layer_lists(wl: Workload, data: dict):
    """A mixed workload as per-layer sequences (W_n, b_n, kind_n), n = 0..N-1: the fully connected layers'
    arrays at n = 0, P, 2P, ..., the convolution layers' arrays elsewhere (pure re-arrangement)."""
    P = wl.fc_period
    Ws, bs, kinds = [], [], []
    for n in range(wl.N):
        if P and n % P == 0:
            Ws.append(data["Wfc"][n // P]); bs.append(data["bfc"][n // P]); kinds.append(FC)
        else:
            Ws.append(data["W"][n]); bs.append(data["b"][n]); kinds.append(CONV)
    return Ws, bs, kinds


def terminal_adjoint(wl: Workload, data: dict, uN: np.ndarray) -> np.ndarray:
    """lambda^N = d(mean cross-entropy)/d u^N for the random softmax head (data preparation
    for the adjoint solve; float64 arithmetic, returned as float32)."""
    B = wl.B
    x = uN.reshape(B, -1).astype(np.float64)
    logits = x @ data["W_o"].astype(np.float64).T
    logits -= logits.max(axis=1, keepdims=True)
    p = np.exp(logits)
    p /= p.sum(axis=1, keepdims=True)
    p[np.arange(B), data["labels"]] -= 1.0
    lam = (p @ data["W_o"].astype(np.float64)) / B
    return lam.reshape(uN.shape).astype(np.float32)


# ---------------------------------------------------------------------------------------------
# The five benchmark workloads and reduced versions of them that the CPU oracle finishes in
# seconds while still spanning several tiles and a ragged tail.
# ---------------------------------------------------------------------------------------------
def cfg1() -> Workload:
    return Workload("cfg1_dense_q8_N16", DENSE, TANH, FP32, N=16, m=4, max_levels=2, relax=RELAX_F,
                    max_iter=4, B=4, q=8, bias_var=0.1)


def cfg2(max_iter: int = 12) -> Workload:
    return Workload("cfg2_dense_q256_N256", DENSE, RELU, FP32, N=256, m=4, max_levels=3,
                    relax=RELAX_FCF, max_iter=max_iter, B=128, q=256, bias_var=0.0)


def cfg3(max_iter: int = 2) -> Workload:
    return Workload("cfg3_conv_c16_28x28_N64", CONV, RELU, FP32, N=64, m=4, max_levels=2,
                    relax=RELAX_FCF, max_iter=max_iter, B=64, C=16, Himg=28, Wimg=28,
                    lifted_input=True)


def cfg4(max_iter: int = 2) -> Workload:
    return Workload("cfg4_conv_c64_32x32_N512", CONV, RELU, BF16, N=512, m=8, max_levels=3,
                    relax=RELAX_FCF, max_iter=max_iter, B=32, C=64, Himg=32, Wimg=32)


def cfg5(max_iter: int = 2) -> Workload:
    return Workload("cfg5_dense_q1024_N1024_train", DENSE, TANH, BF16, N=1024, m=16, max_levels=8,
                    min_coarse=8, relax=RELAX_FCF, max_iter=max_iter, B=256, q=1024,
                    head_classes=10)


def mixed(max_iter: int = 2, dtype: int = FP32) -> Workload:
    """Blocks of one fully connected layer followed by 63 convolution layers (the shape of the paper's second
    training network, Sec. IV-E, at a size one GPU's oracle check can follow); float or bf16 operands."""
    return Workload("mixed_conv_c16_16x16_fc64_N256" + ("_bf16" if dtype == BF16 else ""), CONV, RELU, dtype, N=256,
                    m=4, max_levels=3, relax=RELAX_FCF, max_iter=max_iter, B=32, C=16, Himg=16, Wimg=16, fc_period=64)


def reduced(wl: Workload, **kw) -> Workload:
    """Same structure as `wl` with some fields replaced (smaller N / width / batch)."""
    return dataclasses.replace(wl, **kw)


ALL = {"cfg1": cfg1, "cfg2": cfg2, "cfg3": cfg3, "cfg4": cfg4, "cfg5": cfg5}
