"""Shared helpers of the GPU parity tests: expected values always come from `oracle/`."""
import numpy as np

from oracle import pb_oracle as po


def oracle_reference(W, bits, X, bits_used, frac_bits=16, act_bits=32, rows=None):
    """Oracle results for one layer: dict(q, d, scales, A [m,N,R] int64, Y [N,R] fp32).
    Uses the packed-word tier (pinned against the byte-per-bit tier and numpy in test_oracle.py)."""
    prep = po.prepare(W, bits)
    lw = po.pack_words(prep["layers"])
    R, C = W.shape
    r0, r1 = (0, R) if rows is None else rows
    A, Y = po.matmul_words(lw, prep["scales"], bits_used, C, X, r0=r0, r1=r1, frac_bits=frac_bits,
                           act_bits=act_bits)
    prep.update(A=A, Y=Y, layers_w=lw)
    return prep


def assert_y_close(y_gpu, y_ref, A_ref, scales, frac_bits=16, rtol=1e-5):
    """fp32 outputs: within rtol relative; where layers cancel, relative to the size of the terms
    (both sides sum the per-layer terms in fp64, so they may differ by fp64 rounding of those terms)."""
    y_gpu = np.asarray(y_gpu, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    m = A_ref.shape[0]
    terms = np.zeros_like(y_ref)
    for i in range(m):
        terms += np.abs(float(scales[i]) * A_ref[i].astype(np.float64)) * 2.0 ** -frac_bits
    tol = rtol * np.abs(y_ref) + 1e-12 * terms + 1e-45
    bad = np.abs(y_gpu - y_ref) > tol
    assert not bad.any(), "fp32 mismatch at %s: gpu %s ref %s" % (
        np.argwhere(bad)[:5].tolist(), y_gpu[bad][:5], y_ref[bad][:5])


def pair_sums(A, bits_used):
    """What the matrix-core kernel accumulates when it multiplies two bitlayers at once, from the oracle's
    per-bitlayer sums A [m, N, R]: -2 A[0] + A[1] for the sign pair, 2 A[2p] + A[2p+1] for the others, a last
    single bitlayer if bits_used is odd."""
    m = bits_used
    out = []
    for p in range((m + 1) // 2):
        if 2 * p + 1 <= m - 1:
            out.append((-2 if p == 0 else 2) * A[2 * p] + A[2 * p + 1])
        else:
            out.append(A[m - 1])
    return np.stack(out)
