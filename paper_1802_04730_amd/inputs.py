"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds no arithmetic of the method: it only draws random tensors.
Both the CPU oracle's tests and the GPU path's tests/benchmark take their
inputs from here, so both sides see bit-identical float32 values.

Recipe: ``numpy.random.default_rng(seed)`` (PCG64), each tensor drawn in
float64 in the order listed and then cast to float32.  The default seed of
benchmark configuration c (1..5) is ``180204730 + c``.  Every second
parameter of a normal law is a standard deviation.

The paper uses no public dataset for these operators: the tbmm sizes come from
Factorization Machines (Section 7, transposed batched matmul), the grouped
convolution from ResNeXt-style layers (Section 7, grouped convolutions) and
the MLP from a production model whose layer widths are not published
(Section 7, production models; only the batch size 128 is stated).
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 180204730

# The five benchmark configurations (index 1..5; 0 is unused).
CONFIGS = {
    1: dict(op="tbmm", B=8, N=26, M=72, K=26),
    2: dict(op="tbmm", B=500, N=26, M=72, K=26),
    3: dict(op="mlp", batch=128, dims=(1024, 1024, 512, 256)),
    4: dict(op="gconv", N=32, G=32, C=16, F=16, H=58, W=58, KH=3, KW=3),
    5: dict(op="kron", B=256, I=64, K=64, J=64, L=64),
}


def _rng(seed):
    return np.random.default_rng(seed)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def make_tbmm(B, N, M, K, seed=SEED_BASE + 2):
    """X [B,N,K], Y [B,M,K], i.i.d. uniform[-1,1]."""
    r = _rng(seed)
    X = _f32(r.uniform(-1.0, 1.0, size=(B, N, K)))
    Y = _f32(r.uniform(-1.0, 1.0, size=(B, M, K)))
    return X, Y


def make_mlp(batch, dims, seed=SEED_BASE + 3, w_std=0.02, b_std=0.01):
    """I [batch,dims[0]] ~ N(0,1); then per layer W_l [dims[l+1],dims[l]] ~ N(0,w_std)
    and bias_l [dims[l+1]] ~ N(0,b_std)."""
    r = _rng(seed)
    I = _f32(r.normal(0.0, 1.0, size=(batch, dims[0])))
    Ws, bs = [], []
    for l in range(len(dims) - 1):
        Ws.append(_f32(r.normal(0.0, w_std, size=(dims[l + 1], dims[l]))))
        bs.append(_f32(r.normal(0.0, b_std, size=(dims[l + 1],))))
    return I, Ws, bs


def make_gconv(N, G, C, F, H, W, KH, KW, seed=SEED_BASE + 4, w_std=0.05, b_std=0.05):
    """I [N,G,C,H,W] ~ N(0,1); W1 [G,F,C,KH,KW] ~ N(0,w_std); bias [G*F] ~ N(0,b_std)."""
    r = _rng(seed)
    I = _f32(r.standard_normal(size=(N, G, C, H, W)))
    W1 = _f32(r.normal(0.0, w_std, size=(G, F, C, KH, KW)))
    bias = _f32(r.normal(0.0, b_std, size=(G * F,)))
    return I, W1, bias


def make_kron(B, I, K, J, L, seed=SEED_BASE + 5, std=0.125):
    """W1 [I,K], W2 [J,L], X [B,K,L], all ~ N(0,std)."""
    r = _rng(seed)
    W1 = _f32(r.normal(0.0, std, size=(I, K)))
    W2 = _f32(r.normal(0.0, std, size=(J, L)))
    X = _f32(r.normal(0.0, std, size=(B, K, L)))
    return W1, W2, X


def make_sconv2d(N, C, F, H, W, KH, KW, seed=SEED_BASE + 6, w_std=0.05, b_std=0.05):
    """I [N,C,H,W] ~ N(0,1); W [F,C,KH,KW] ~ N(0,w_std); bias [F] ~ N(0,b_std) (Section 3, listing sconv2d; the
    paper states no sizes or distributions for it: those of the grouped convolution are reused)."""
    r = _rng(seed)
    I = _f32(r.standard_normal(size=(N, C, H, W)))
    Wt = _f32(r.normal(0.0, w_std, size=(F, C, KH, KW)))
    bias = _f32(r.normal(0.0, b_std, size=(F,)))
    return I, Wt, bias


def make_lut(E, D, B, L, seed=SEED_BASE + 7):
    """LUT [E,D] ~ N(0,1), drawn directly in float32 (at the paper's E = 10^7 a float64 draw would need 5 GB);
    Idx [B,L] int32, uniform over [0,E) with repetitions allowed.  The paper's production indices are not
    published (Section 7, production models); uniform random rows stand in for them."""
    r = _rng(seed)
    LUT = r.standard_normal(size=(E, D), dtype=np.float32)
    Idx = r.integers(0, E, size=(B, L), dtype=np.int32)
    return LUT, Idx


def make_lut_indices(E, B, L, seed):
    """Idx [B,L] int32 alone, uniform over [0,E) (a second table's lookups without a second table draw)."""
    return _rng(seed).integers(0, E, size=(B, L), dtype=np.int32)


def make_config(c):
    """Inputs of benchmark configuration c (1..5) with its default seed."""
    cfg = dict(CONFIGS[c])
    op = cfg.pop("op")
    seed = SEED_BASE + c
    if op == "tbmm":
        return op, make_tbmm(seed=seed, **cfg)
    if op == "mlp":
        return op, make_mlp(seed=seed, **cfg)
    if op == "gconv":
        return op, make_gconv(seed=seed, **cfg)
    if op == "kron":
        return op, make_kron(seed=seed, **cfg)
    raise KeyError(op)


# Algorithmic work per configuration: one multiply + one add per contraction
# term; each input read once and each declared output written once (fp32).
def flops_tbmm(B, N, M, K):
    return 2 * B * N * M * K


def bytes_tbmm(B, N, M, K):
    return 4 * (B * N * K + B * M * K + B * N * M)


def flops_mlp(batch, dims):
    return sum(2 * batch * dims[l] * dims[l + 1] for l in range(len(dims) - 1))


def bytes_mlp(batch, dims):
    n = batch * dims[0]
    for l in range(len(dims) - 1):
        n += dims[l] * dims[l + 1] + dims[l + 1] + batch * dims[l + 1]
    return 4 * n


def flops_gconv(N, G, C, F, H, W, KH, KW):
    return 2 * N * G * F * (H - KH + 1) * (W - KW + 1) * C * KH * KW


def bytes_gconv(N, G, C, F, H, W, KH, KW):
    return 4 * (N * G * C * H * W + G * F * C * KH * KW + G * F
                + N * G * F * (H - KH + 1) * (W - KW + 1))


def flops_kron(B, I, K, J, L):
    # two-stage evaluation: T = W1 . X_b (2*I*K*L), Y_b = T . W2^T (2*I*J*L)
    return 2 * B * I * K * L + 2 * B * I * J * L


def bytes_kron(B, I, K, J, L):
    return 4 * (I * K + J * L + B * K * L + B * I * J)


def flops_sconv2d(N, C, F, H, W, KH, KW, sh, sw):
    return 2 * N * F * ((H - KH) // sh + 1) * ((W - KW) // sw + 1) * C * KH * KW


def bytes_sconv2d(N, C, F, H, W, KH, KW, sh, sw):
    return 4 * (N * C * H * W + F * C * KH * KW + F + N * F * ((H - KH) // sh + 1) * ((W - KW) // sw + 1))


def flops_lut(E, D, B, L):
    return B * D * L  # one addition per gathered element


def bytes_lut(E, D, B, L):
    # the gathered rows, the indices, the output; the table as a whole is never read
    return 4 * (B * L * D + B * L + B * D)
