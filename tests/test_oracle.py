"""Pins for the CPU oracle: everything here checks `oracle/` against something
other than itself -- values the paper prints, closed forms, numpy's integer
matmul as brute force, exact rational arithmetic, a library LSTM cell."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import pb_oracle as po
from paper_2003_00822_amd import synth


# --------------------------------------------------------------------------
# Supplementary material, "Detailed Example of Precision Batching": printed values
# --------------------------------------------------------------------------
def test_worked_example_bitlayers_and_scales(golden_example):
    g = golden_example
    q = np.array(g["W"], dtype=np.int32).reshape(2, 2)
    layers, s = po.bitlayers(q, 4)
    for i, name in enumerate(["W1", "W2", "W3", "W4"]):
        assert layers[i].reshape(-1).tolist() == g[name], name
    assert s.tolist() == g["S"]
    # "Verify that W = sum_i W_i S_i"
    assert (np.tensordot(s, layers.astype(np.int64), axes=1) == q).all()


def test_worked_example_planes(golden_example):
    g = golden_example
    xq = np.array(g["x"], dtype=np.int32)
    pl, c = po.planes(xq, act_bits=4)
    # printed x^(b): one row per element, MSB first; oracle planes: [plane j (LSB=0)][element]
    xb = np.array(g["XB"]).reshape(2, 4)
    assert (pl[::-1].T == xb).all()
    assert c[::-1].tolist() == g["SX"]
    # "Verify that x = x^(b) S_x"
    assert (xb @ np.array(g["SX"]) == xq).all()


def test_worked_example_product(golden_example):
    g = golden_example
    # a third row [7, 0] makes max|W| = 7 = qmax, hence d = 1 and q == W under the symmetric quantizer
    W = np.array([[1, -1], [4, -4], [7, 0]], dtype=np.float32)
    prep = po.prepare(W, 4)
    assert prep["d"] == 1.0
    assert (prep["q"][:2].reshape(-1) == np.array(g["W"])).all()
    x = np.array([g["x"]], dtype=np.float32)
    # integers as in the example: fixed point at 2^0, 4 activation planes
    A, T, Y = po.matmul_bitserial(prep["layers"], prep["scales"], prep["s"], 4, x, frac_bits=0, act_bits=4)
    # W x = [1*1 + (-1)(-2), 4*1 + (-4)(-2)] = [3, 12]
    assert T[0, :2].tolist() == [3, 12]
    assert Y[0, :2].tolist() == [3.0, 12.0]
    # per-bitlayer products W_i x for the printed layers: [-2,-2], [-2,-1], [-2,0], [-1,0]
    assert A[:, 0, :2].tolist() == [[-2, -2], [-2, -1], [-2, 0], [-1, 0]]
    # accumulating only the first m layers = dropping W's low bits: [16,16], [8,12], [4,12], [3,12]
    want = [[16, 16], [8, 12], [4, 12], [3, 12]]
    for m in range(1, 5):
        _, Tm, Ym = po.matmul_bitserial(prep["layers"], prep["scales"], prep["s"], m, x, frac_bits=0, act_bits=4)
        assert Tm[0, :2].tolist() == want[m - 1]
        assert Ym[0, :2].tolist() == [float(v) for v in want[m - 1]]
    # same with the 32-bit, 16-fraction-bit format of Algorithm 2
    _, T32, Y32 = po.matmul_bitserial(prep["layers"], prep["scales"], prep["s"], 4, x)
    assert T32[0, :2].tolist() == [3 << 16, 12 << 16]
    assert Y32[0, :2].tolist() == [3.0, 12.0]


# --------------------------------------------------------------------------
# Section 3.2: two's-complement decomposition, exhaustive
# --------------------------------------------------------------------------
@pytest.mark.parametrize("bits", list(range(1, 9)) + [12, 16])
def test_bitlayers_reconstruct_all_codes(bits):
    q = np.arange(-(1 << (bits - 1)), 1 << (bits - 1), dtype=np.int32)
    layers, s = po.bitlayers(q, bits)
    assert set(np.unique(layers).tolist()) <= {0, 1}
    assert s[0] == -(1 << (bits - 1))
    assert s[1:].tolist() == [1 << (bits - 1 - i) for i in range(1, bits)]
    assert (np.tensordot(s, layers.astype(np.int64), axes=1) == q).all()
    # range statement of Section 3.2: n magnitude layers + sign cover [-2^n, 2^n - 1]
    n = bits - 1
    assert q.min() == -(2 ** n) and q.max() == 2 ** n - 1


@pytest.mark.parametrize("k", [2, 4, 8, 16, 32])
def test_planes_reconstruct(k):
    rng = np.random.default_rng(k)
    lo, hi = -(1 << (k - 1)), (1 << (k - 1)) - 1
    xq = rng.integers(lo, hi + 1, size=300, dtype=np.int64)
    xq[:3] = [lo, hi, -1]
    xq = xq.astype(np.int32)
    pl, c = po.planes(xq, act_bits=k)
    assert c[k - 1] == -(1 << (k - 1))
    assert c[: k - 1].tolist() == [1 << j for j in range(k - 1)]
    assert (c @ pl.astype(np.int64) == xq).all()


# --------------------------------------------------------------------------
# Section 3.1 identity: bit-serial product == integer matmul (numpy as brute force)
# --------------------------------------------------------------------------
def _truncate(q, bits, m):
    sh = bits - m
    return (q.astype(np.int64) >> sh) << sh


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 5, 8])
@pytest.mark.parametrize("shape", [(3, 5), (7, 33), (16, 64), (5, 96), (64, 96)])
def test_bitserial_equals_integer_matmul(bits, shape):
    R, C = shape
    rng = np.random.default_rng(100 * bits + R + C)
    q = rng.integers(-(1 << (bits - 1)), 1 << (bits - 1), size=(R, C)).astype(np.int32)
    layers, s = po.bitlayers(q, bits)
    X = (rng.normal(0, 1.5, size=(3, C)) * np.exp2(rng.integers(-8, 6, size=(3, C)))).astype(np.float32)
    xq = po.fixed_point(X)
    sc = po.scales(0.37, bits)
    for m in range(1, bits + 1):
        A, T, Y = po.matmul_bitserial(layers, sc, s, m, X)
        for i in range(m):
            assert (A[i] == xq.astype(np.int64) @ layers[i].astype(np.int64).T).all()
        assert (T == xq.astype(np.int64) @ _truncate(q, bits, m).T).all()
        # direct definition in the oracle agrees too
        assert (po.layer_products_direct(layers, m, xq) == A).all()


def test_bitserial_exhaustive_tiny():
    # every 2-bit 2x2 weight matrix against every 3-bit activation pair
    bits, k = 2, 3
    codes = range(-2, 2)
    acts = range(-4, 4)
    for a in codes:
        for b in codes:
            for c_ in codes:
                for d in codes:
                    q = np.array([[a, b], [c_, d]], dtype=np.int32)
                    layers, s = po.bitlayers(q, bits)
                    X = np.array([[u, v] for u in acts for v in acts], dtype=np.float32)
                    _, T, _ = po.matmul_bitserial(layers, po.scales(1.0, bits), s, bits, X, frac_bits=0, act_bits=k)
                    assert (T == X.astype(np.int64) @ q.astype(np.int64).T).all()


def test_special_activation_vectors():
    bits, R, C = 5, 9, 70  # C not a multiple of 32 or 64: padding must contribute nothing
    rng = np.random.default_rng(5)
    q = rng.integers(-16, 16, size=(R, C)).astype(np.int32)
    layers, s = po.bitlayers(q, bits)
    sc = po.scales(1.0, bits)
    # one-hot activation reads a column of each bitlayer back
    for col, val in [(0, 3.25), (31, -1.0), (32, 0.5), (69, -7.0)]:
        X = np.zeros((1, C), dtype=np.float32)
        X[0, col] = val
        A, T, _ = po.matmul_bitserial(layers, sc, s, bits, X)
        v = int(val * 65536)
        for i in range(bits):
            assert (A[i, 0] == v * layers[i][:, col].astype(np.int64)).all()
        assert (T[0] == v * q[:, col].astype(np.int64)).all()
    # x_q = -1 everywhere: all 32 planes are all-ones, A_i = -rowpopcount
    X = np.full((1, C), -1.0 / 65536, dtype=np.float32)
    assert (po.fixed_point(X) == -1).all()
    A, _, _ = po.matmul_bitserial(layers, sc, s, bits, X)
    for i in range(bits):
        assert (A[i, 0] == -layers[i].sum(axis=1).astype(np.int64)).all()
    # x_q = INT32_MIN everywhere: only the negative top plane is set
    X = np.full((1, C), -40000.0, dtype=np.float32)
    assert (po.fixed_point(X) == -(2 ** 31)).all()
    A, _, _ = po.matmul_bitserial(layers, sc, s, bits, X)
    for i in range(bits):
        assert (A[i, 0] == -(2 ** 31) * layers[i].sum(axis=1).astype(np.int64)).all()


def test_word_level_tier_matches_definition_level():
    for (R, C, bits) in [(5, 1, 3), (9, 63, 4), (17, 64, 8), (12, 65, 2), (33, 200, 6)]:
        W, X = synth.ragged(R, C, batch=2, case=bits, xdist="wide")
        prep = po.prepare(W, bits)
        lw = po.pack_words(prep["layers"])
        assert lw.shape == (bits, R, (C + 63) // 64)
        for m in (1, bits):
            A, T, Y = po.matmul_bitserial(prep["layers"], prep["scales"], prep["s"], m, X)
            Aw, Yw = po.matmul_words(lw, prep["scales"], m, C, X)
            assert (A == Aw).all()
            assert (Y.view(np.int32) == Yw.view(np.int32)).all()
        # row range restriction
        Aw2, Yw2 = po.matmul_words(lw, prep["scales"], bits, C, X, r0=2, r1=4)
        assert (Aw2[:, :, 2:4] == A[:, :, 2:4]).all() and (Aw2[:, :, :2] == 0).all()


def test_pack_words_bit_positions():
    b = np.zeros((2, 130), dtype=np.uint8)
    b[0, 0] = 1
    b[0, 63] = 1
    b[0, 64] = 1
    b[1, 129] = 1
    w = po.pack_words(b)
    assert w.shape == (2, 3)
    assert w[0].tolist() == [(1 << 63) | 1, 1, 0]
    assert w[1].tolist() == [0, 0, 2]


# --------------------------------------------------------------------------
# Section 3.3 quantizer: invariants (no values printed in the paper: parity unpinned beyond these)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_quantizer_invariants(bits):
    rng = np.random.default_rng(bits)
    W = rng.normal(0, 0.05, size=(40, 50)).astype(np.float32)
    q, d = po.quantize(W, bits)
    qmax = (1 << (bits - 1)) - 1
    M = np.abs(W).max()
    assert d == np.float32(M) / np.float32(qmax)
    assert q.max() <= qmax and q.min() >= -qmax - 1
    # the largest-magnitude element maps to +-qmax
    i = np.unravel_index(np.abs(W).argmax(), W.shape)
    assert abs(int(q[i])) == qmax
    # nearest grid point: |W - d q| <= d/2 (plus fp32 rounding of the quotient)
    err = np.abs(W.astype(np.float64) - float(d) * q)
    assert err.max() <= float(d) * (0.5 + 1e-6)
    # monotone
    order = np.argsort(W.reshape(-1), kind="stable")
    assert (np.diff(q.reshape(-1)[order]) >= 0).all()
    # idempotent on the dequantized values
    Wd = (np.float32(d) * q.astype(np.float32)).astype(np.float32)
    q2, d2 = po.quantize(Wd, bits)
    assert (q2 == q).all()


def test_quantizer_ties_and_degenerate():
    # ties go to even: W/d = 0.5, 1.5, 2.5, -0.5, -1.5 with d = 1 (max|W| = 7 = qmax at 4 bits)
    W = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 7.0], dtype=np.float32)
    q, d = po.quantize(W, 4)
    assert d == 1.0
    assert q.tolist() == [0, 2, 2, 0, -2, -2, 7]
    # all-zero matrix
    q, d = po.quantize(np.zeros(5, dtype=np.float32), 4)
    assert d == 1.0 and (q == 0).all()
    # 1 bit: only the sign layer, codes {-1, 0}, d = max|W|
    W = np.array([0.2, -0.2, -0.09, -0.11, 0.0], dtype=np.float32)
    q, d = po.quantize(W, 1)
    assert d == np.float32(0.2)
    assert q.tolist() == [0, -1, 0, -1, 0]
    sc = po.scales(d, 1)
    assert sc.tolist() == [-np.float32(0.2)]
    # scales are d times the integer ladder, sign layer negative
    sc = po.scales(np.float32(0.375), 4)
    assert sc.tolist() == [-3.0, 1.5, 0.75, 0.375]


# --------------------------------------------------------------------------
# Section 3.3 / Algorithm 2: activations to 32-bit fixed point by multiply and cast
# --------------------------------------------------------------------------
def test_fixed_point_hand_values():
    u = 2.0 ** -16
    cases = [
        (0.0, 0), (1.0, 65536), (-2.0, -131072),
        (0.5 * u, 0), (-0.5 * u, 0),              # truncation is toward zero, both signs
        (1.5 * u, 1), (-1.5 * u, -1),
        (1.0 - 2.0 ** -24, 65535),                # 65535.996 truncates down
        (-(1.0 - 2.0 ** -24), -65535),
        (32767.998046875, 2147483520),            # largest fp32 below 2^15
        (32768.0, 2 ** 31 - 1),                   # saturates
        (-32768.0, -(2 ** 31)),
        (-32768.5, -(2 ** 31)),
        (1e30, 2 ** 31 - 1), (-1e30, -(2 ** 31)),
        (float("inf"), 2 ** 31 - 1), (float("-inf"), -(2 ** 31)),
        (float("nan"), 0),
    ]
    x = np.array([c[0] for c in cases], dtype=np.float32)
    got = po.fixed_point(x).tolist()
    assert got == [c[1] for c in cases]
    # other fixed-point positions and widths (the fixed point "may be changed", Section 3.1)
    assert po.fixed_point(np.array([1.75, -1.75], dtype=np.float32), frac_bits=1).tolist() == [3, -3]
    assert po.fixed_point(np.array([3.0, 200.0, -200.0], dtype=np.float32), frac_bits=4, act_bits=8).tolist() == [48, 127, -128]


def test_fixed_point_matches_exact_arithmetic():
    rng = np.random.default_rng(11)
    x = (rng.normal(size=2000) * np.exp2(rng.integers(-30, 18, size=2000))).astype(np.float32)
    got = po.fixed_point(x)
    for xi, gi in zip(x.tolist(), got.tolist()):
        t = Fraction(xi) * 65536
        t = int(t) if t >= 0 else -int(-t)  # toward zero
        t = max(-(2 ** 31), min(2 ** 31 - 1, t))
        assert gi == t


# --------------------------------------------------------------------------
# Algorithm 2's scaling: fp32 output vs exact rational arithmetic
# --------------------------------------------------------------------------
def test_dequant_against_exact_rationals():
    rng = np.random.default_rng(3)
    bits = 8
    A = rng.integers(-(2 ** 44), 2 ** 44, size=(bits, 64)).astype(np.int64)
    sc = po.scales(np.float32(0.0123), bits)
    for m in (1, 3, 8):
        y = po.dequant(A, sc, m)
        for r in range(64):
            exact = sum(Fraction(float(sc[i])) * int(A[i, r]) for i in range(m)) / 65536
            ref = np.float32(float(exact))
            scale = sum(abs(Fraction(float(sc[i])) * int(A[i, r])) for i in range(m)) / 65536
            assert abs(float(y[r]) - float(exact)) <= 1e-6 * float(scale) + abs(float(ref)) * 1e-7


def test_output_close_to_full_precision_product():
    # sanity, not parity: with all layers the result approximates W x within the quantization error bound
    W, X = synth.ragged(48, 200, batch=2, case=1, std=0.05, xdist="uniform")
    bits = 8
    prep = po.prepare(W, bits)
    _, _, Y = po.matmul_bitserial(prep["layers"], prep["scales"], prep["s"], bits, X)
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    d = float(prep["d"])
    bound = 0.5 * d * np.abs(X).sum(axis=1, keepdims=True) + 2.0 ** -16 * np.abs(d * prep["q"]).sum(axis=1)[None, :]
    assert (np.abs(Y - ref) <= bound + 1e-6).all()
    # fewer layers: error grows monotonically on average
    errs = []
    for m in range(1, bits + 1):
        _, _, Ym = po.matmul_bitserial(prep["layers"], prep["scales"], prep["s"], m, X)
        errs.append(np.abs(Ym - ref).mean())
    assert errs[-1] < errs[3] < errs[0]


# --------------------------------------------------------------------------
# LSTM cell pointwise part against a library routine
# --------------------------------------------------------------------------
def test_lstm_pointwise_matches_torch_cell():
    torch = pytest.importorskip("torch")
    H, I, N = 7, 5, 3
    rng = np.random.default_rng(2)
    Wg = rng.uniform(-0.5, 0.5, size=(4 * H, I + H))
    b = rng.uniform(-0.2, 0.2, size=4 * H)
    x = rng.normal(size=(N, I))
    h0 = rng.uniform(-1, 1, size=(N, H))
    c0 = rng.normal(size=(N, H))
    cell = torch.nn.LSTMCell(I, H).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(Wg[:, :I]))
        cell.weight_hh.copy_(torch.from_numpy(Wg[:, I:]))
        cell.bias_ih.copy_(torch.from_numpy(b))
        cell.bias_hh.zero_()
        h1, c1 = cell(torch.from_numpy(x), (torch.from_numpy(h0), torch.from_numpy(c0)))
    gates = (np.concatenate([x, h0], axis=1) @ Wg.T).astype(np.float32)
    h, c = po.lstm_pointwise(gates, b.astype(np.float32), c0.astype(np.float32))
    assert np.abs(h - h1.numpy()).max() < 2e-6
    assert np.abs(c - c1.numpy()).max() < 2e-6


# ---------------------------------------------------------------------------------------------------------------
# Section 3.3's other quantizers (oracle readings; the paper prints no values: closed forms, brute force, invariants)

def test_range_quantizer_hand_values():
    # d = (max - min) / 2^n with n = B - 1: W = [-1, 0, 1, 3], B = 3 -> d = 1, codes = W
    W = np.array([-1.0, 0.0, 1.0, 3.0], dtype=np.float32)
    q, d = po.quantize_mode(W, 3, po.QUANT_RANGE)
    assert d == 1.0 and q.tolist() == [-1, 0, 1, 3]
    # B = 2 -> d = 2: W / d = [-0.5, 0, 0.5, 1.5] -> round half to even [0, 0, 0, 2], clamped to the code range [-2, 1]
    q, d = po.quantize_mode(W, 2, po.QUANT_RANGE)
    assert d == 2.0 and q.tolist() == [0, 0, 0, 1]
    # one-signed weights overflow the range and are clamped (the reason the default quantizer is symmetric)
    W = np.array([0.0, 1.0, 2.0, 3.0, 4.0], dtype=np.float32)
    q, d = po.quantize_mode(W, 3, po.QUANT_RANGE)
    assert d == 1.0 and q.tolist() == [0, 1, 2, 3, 3]
    # constant matrix: d = 1
    q, d = po.quantize_mode(np.full(5, 0.25, dtype=np.float32), 4, po.QUANT_RANGE)
    assert d == 1.0 and q.tolist() == [0] * 5


def test_sign_quantizer_hand_values_and_mean():
    W = np.array([0.5, -1.5, 2.0, -4.0], dtype=np.float32)
    q, d = po.quantize_mode(W, 2, po.QUANT_SIGN)
    assert q.tolist() == [1, -1, 1, -1] and d == 2.0            # mean |W| = 8 / 4
    layers, s = po.bitlayers(q, 2)
    assert s.tolist() == [-2, 1]
    assert layers.tolist() == [[0, 1, 0, 1], [1, 1, 1, 1]]       # +1 = (0, 1), -1 = (1, 1): no code is 0
    with pytest.raises(ValueError):
        po.quantize_mode(W, 3, po.QUANT_SIGN)
    rng = np.random.default_rng(5)
    W = rng.normal(0, 0.05, size=5000).astype(np.float32)
    q, d = po.quantize_mode(W, 2, po.QUANT_SIGN)
    assert set(np.unique(q).tolist()) == {-1, 1} and (q == np.where(W >= 0, 1, -1)).all()
    exact = np.abs(W.astype(np.float64)).mean()
    assert abs(float(d) - exact) <= 2.0 ** -28 * np.abs(W).max() + 1e-7 * exact    # truncation to 2^(e-30) per term
    # the least-squares property of that scale: no other scale has a smaller squared error
    err = lambda t: ((W.astype(np.float64) - t * q) ** 2).sum()
    assert err(float(d)) <= min(err(float(d) * 1.01), err(float(d) * 0.99))


def test_clip_search_worked_by_hand():
    """Section 3.3's clipping search on a case small enough to do on paper.  W = [32, 6, -6, 6, -6, 5, -5], B = 2:
    codes -2 .. 1, thresholds T_k = 32 k / 32 = k, step d_k = T_k / 1 = k, error = sum |W - d q| (mean x 7).
    The 32 always gets code 1 (error 32 - k); for the six small weights:
      k = 6: 6 -> 1, -6 -> -1 (0 each); 5 -> 1, -5 -> -1 (1 each)                    26 + 0 + 2 = 28   <- smallest
      k = 5: +-6 -> +-1 (1 each, four of them); +-5 -> +-1 (0)                       27 + 4 + 0 = 31   runner-up
      k = 7: +-6 -> +-1 (1 each); +-5 -> +-1 (2 each)                                25 + 4 + 4 = 33
      k = 4: 6 / 4 = 1.5 -> 2 (half to even), clamped to 1 (2 each); -6 -> -2 (2 each); +-5 -> +-1 (1 each)
                                                                                    28 + 8 + 2 = 38
      k = 3: 6 -> 2 -> clamped 1 (3 each); -6 -> -2 (0); 5 -> 2 -> 1 (2); -5 -> -2 (1)   29 + 6 + 3 = 38
      k >= 12: all six round to 0                                                   (32 - k) + 34, 34 at k = 32
    so clipping at T = 6 wins with step 6 and codes [1, 1, -1, 1, -1, 1, -1].
    With squared errors the unclipped k = 32 would win (194 against 678 at k = 6): the measure is the absolute error."""
    W = np.array([32, 6, -6, 6, -6, 5, -5], dtype=np.float32)
    q, d = po.quantize_mode(W, 2, po.QUANT_CLIP)
    assert d == 6.0 and q.tolist() == [1, 1, -1, 1, -1, 1, -1]
    # the same weights scaled by 2^-7 (all values stay exact): the step scales, the codes stay
    q, d = po.quantize_mode(W * np.float32(2.0 ** -7), 2, po.QUANT_CLIP)
    assert d == 6.0 * 2.0 ** -7 and q.tolist() == [1, 1, -1, 1, -1, 1, -1]


def test_clip_search_tie_takes_the_larger_threshold():
    """W = [32, -10, 2, 9, 4, -9], B = 2 (step d_k = k):
      k = 10: 22 + |-10 + 10| + 2 + |9 - 10| + 4 + |-9 + 10| = 22 + 0 + 2 + 1 + 4 + 1 = 30
      k =  9: 23 + |-10 +  9| + 2 + |9 -  9| + 4 + |-9 +  9| = 23 + 1 + 2 + 0 + 4 + 0 = 30
      k = 11: 21 + 1 + 2 + 2 + 4 + 2 = 32, every other k is larger still (34 at k = 32).
    Two thresholds tie exactly; the reading keeps the larger one (the one that clips less)."""
    W = np.array([32, -10, 2, 9, 4, -9], dtype=np.float32)
    q, d = po.quantize_mode(W, 2, po.QUANT_CLIP)
    assert d == 10.0 and q.tolist() == [1, -1, 0, 1, 0, -1]


def _exact_clip_errors(W, bits):
    """sum |W - d_k q| for k = 1 .. 32 in exact rational arithmetic; d_k is the fp32 step of threshold max|W| k / 32,
    q = round-half-even(W / d_k) clamped to the B-bit codes."""
    from fractions import Fraction as Fr
    f32 = np.float32
    M = f32(np.abs(W).max())
    qmax, qmin = (1 << (bits - 1)) - 1, -(1 << (bits - 1))
    out = {}
    for k in range(1, 33):
        d32 = f32(f32(M * f32(k / 32.0)) / f32(max(qmax, 1)))
        d = Fr(float(d32))
        E = Fr(0)
        for w in W:
            w = Fr(float(w))
            t = w / d
            fl = t.numerator // t.denominator
            r = t - fl
            qq = fl + 1 if r > Fr(1, 2) else fl if r < Fr(1, 2) else (fl if fl % 2 == 0 else fl + 1)
            # (the oracle rounds the fp32 quotient; a quotient within half an ulp of a tie may round the other way,
            # which changes |W - d q| by at most 2^-23 |W|: inside the slack of the caller)
            qq = min(max(qq, qmin), qmax)
            E += abs(w - d * qq)
        out[k] = (E, d32)
    return out


@pytest.mark.parametrize("bits,seed", [(2, 1), (3, 2), (4, 3), (5, 4), (8, 5)])
def test_clip_search_minimises_the_exact_mean_absolute_error(bits, seed):
    """The winner's exact error is the smallest of the 32 candidates' exact errors, up to what the oracle's own
    arithmetic loses: fp32 rounding of each product and difference (2^-23 of max|W| per element, twice) and the
    truncation of each term to a multiple of 2^(e-30)."""
    from fractions import Fraction as Fr
    rng = np.random.default_rng(400 + seed)
    W = rng.normal(0, 0.05, size=300).astype(np.float32)
    W[11] = 0.9                                                  # an outlier: clipping pays off
    q, d = po.quantize_mode(W, bits, po.QUANT_CLIP)
    errs = _exact_clip_errors(W, bits)
    mine = [k for k, (E, d32) in errs.items() if d32 == d]
    assert mine, "the step is not one of the 32 candidates"
    k_star = max(mine)
    slack = Fr(len(W)) * Fr(float(np.abs(W).max())) * Fr(3, 2 ** 23)
    best = min(E for E, _ in errs.values())
    assert errs[k_star][0] <= best + slack
    if 3 <= bits <= 5:
        assert k_star < 32                                        # the outlier is clipped (a coarse grid gains from it)
    # codes are those of the symmetric quantizer with that step
    qmax, qmin = (1 << (bits - 1)) - 1, -(1 << (bits - 1))
    q_ref = np.clip(np.rint((W / d).astype(np.float32)), qmin, qmax).astype(np.int32)
    assert (q == q_ref).all()
    # a different objective or candidate set would not pass: the squared-error optimum and the unclipped step differ
    q0, d0 = po.quantize(W, bits)
    mae = lambda qq, dd: np.abs(W.astype(np.float64) - float(dd) * qq).mean()
    if 3 <= bits <= 5:
        assert mae(q, d) < mae(q0, d0)
    else:
        assert mae(q, d) <= mae(q0, d0)


def test_clip_search_invariances():
    """Order of the weights does not matter (the error sums are exact integers); scaling by 2^p scales the step by 2^p
    and leaves the codes."""
    rng = np.random.default_rng(77)
    W = rng.normal(0, 0.05, size=500).astype(np.float32)
    W[3] = -1.25
    for bits in (2, 4, 7):
        q, d = po.quantize_mode(W, bits, po.QUANT_CLIP)
        perm = rng.permutation(W.size)
        qp, dp = po.quantize_mode(W[perm], bits, po.QUANT_CLIP)
        assert dp == d and (qp == q[perm]).all()
        for p in (-9, 5):
            qs, ds = po.quantize_mode((W * np.float32(2.0 ** p)).astype(np.float32), bits, po.QUANT_CLIP)
            assert ds == np.float32(d * np.float32(2.0 ** p)) and (qs == q).all()
        # the mirror image: the code range is not symmetric (-2^(B-1) .. 2^(B-1) - 1), the threshold search is
        qn, dn = po.quantize_mode(-W, bits, po.QUANT_CLIP)
        assert np.abs(W.astype(np.float64) + float(dn) * qn).mean() <= np.abs(W.astype(np.float64)).mean()


def test_clip_search_keeps_an_exact_grid():
    # weights already on the grid of the unclipped quantizer: zero error at k = 32, nothing smaller exists
    bits = 4
    codes = np.arange(-7, 8, dtype=np.float32)
    W = (codes * np.float32(0.125)).astype(np.float32)
    q, d = po.quantize_mode(W, bits, po.QUANT_CLIP)
    assert d == np.float32(0.125) and (q == codes.astype(np.int32)).all()
    q, d = po.quantize_mode(np.zeros(9, dtype=np.float32), bits, po.QUANT_CLIP)
    assert d == 1.0 and not q.any()


@pytest.mark.parametrize("mode", [1, 2, 3])
def test_quantizer_variants_feed_algorithm_1_unchanged(mode):
    """Whatever the quantizer, bitlayers and scales reconstruct d * q (Section 3.3: any linearly spaced grid)."""
    rng = np.random.default_rng(60 + mode)
    W = rng.normal(0, 0.3, size=(6, 40)).astype(np.float32)
    bits = 2 if mode == 2 else 5
    prep = po.prepare(W, bits, mode)
    rec = np.tensordot(prep["s"], prep["layers"].astype(np.int64), axes=1)
    assert (rec == prep["q"]).all()
    assert np.allclose(prep["scales"], float(prep["d"]) * prep["s"].astype(np.float64), rtol=0, atol=0)
