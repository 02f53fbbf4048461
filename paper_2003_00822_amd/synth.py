"""Seeded synthetic inputs shaped like the paper's FC / MLP / LSTM workloads.

This module holds no arithmetic of the method (no quantization, no bit
decomposition, no products): it only draws random weights and activations.
Both the CPU oracle's tests and the HIP path's tests/benchmarks take their
inputs from here, so that the two sides see identical arrays.

Shapes follow the paper's evaluation: square FC layers of Table 1
(512..4096), the 3-layer fully connected MNIST network with hidden size 4096
(Section 4.2), and LSTM gate matrices (Section 4.2); value distributions are
the ones the benchmark configurations name.  The paper's datasets and trained
weights are not available, so these arrays stand in for them.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 200300822


def _rng(cfg: int, case: int) -> np.random.Generator:
    return np.random.default_rng(BASE_SEED + 1000 * int(cfg) + int(case))


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def fc_small(case: int = 0):
    """Config 1: W 1024x1024 ~N(0,0.05), x 1024 ~U(-1,1), batch 1."""
    g = _rng(1, case)
    W = _f32(g.normal(0.0, 0.05, size=(1024, 1024)))
    X = _f32(g.uniform(-1.0, 1.0, size=(1, 1024)))
    return W, X


def fc_square(n: int = 4096, std: float = 0.02, batch: int = 1, case: int = 0, cfg: int = 2):
    """Config 2 (n=4096, std 0.02) and config 5 (n=8192, std 0.01, batch 1..64):
    W n x n ~N(0,std), X batch x n ~N(0,1)."""
    g = _rng(cfg, case)
    W = _f32(g.normal(0.0, std, size=(n, n)))
    X = _f32(g.normal(0.0, 1.0, size=(batch, n)))
    return W, X


def fc_large(batch: int = 1, case: int = 0):
    """Config 5: W 8192x8192 ~N(0,0.01), X batch x 8192 ~N(0,1)."""
    return fc_square(8192, 0.01, batch, case, cfg=5)


def mlp(case: int = 0):
    """Config 3: 784-4096-4096-10 MLP, weights ~N(0, var=1/fan_in), input ~U(0,1)."""
    g = _rng(3, case)
    dims = [784, 4096, 4096, 10]
    Ws = [_f32(g.normal(0.0, 1.0 / np.sqrt(dims[i]), size=(dims[i + 1], dims[i]))) for i in range(3)]
    X = _f32(g.uniform(0.0, 1.0, size=(1, 784)))
    return Ws, X


def lstm(hidden: int = 1500, inp: int = 1500, steps: int = 35, batch: int = 1, case: int = 0):
    """Config 4: fused gate matrix (4*hidden) x (inp+hidden) ~U(-0.04,0.04),
    inputs x_t ~N(0,1) for `steps` time steps, zero bias, h0 = c0 = 0."""
    g = _rng(4, case)
    W = _f32(g.uniform(-0.04, 0.04, size=(4 * hidden, inp + hidden)))
    xs = _f32(g.normal(0.0, 1.0, size=(steps, batch, inp)))
    bias = np.zeros(4 * hidden, dtype=np.float32)
    return W, xs, bias


def ragged(rows: int, cols: int, batch: int = 1, case: int = 0, std: float = 0.05, xdist: str = "normal"):
    """Arbitrary (ragged) shapes for edge-case tests."""
    g = _rng(9, case + 7 * rows + 13 * cols + 31 * batch)
    W = _f32(g.normal(0.0, std, size=(rows, cols)))
    if xdist == "normal":
        X = _f32(g.normal(0.0, 1.0, size=(batch, cols)))
    elif xdist == "uniform":
        X = _f32(g.uniform(-1.0, 1.0, size=(batch, cols)))
    elif xdist == "relu":
        X = _f32(np.maximum(g.normal(0.0, 1.0, size=(batch, cols)), 0.0))
    elif xdist == "wide":
        # wide dynamic range, including values that saturate the 32-bit fixed point
        X = _f32(g.normal(0.0, 1.0, size=(batch, cols)) * np.exp2(g.integers(-20, 17, size=(batch, cols))))
    else:
        raise ValueError(xdist)
    return W, X
