"""Worst-case sizes of the partial sums of the matrix-core kernel (csrc/pb_mfma.hip), worked out on the host.

The kernel keeps the exact integer A_i[r] = sum_c bit_i[r, c] * x_q[c] of Algorithm 2 in narrower pieces: fp32
accumulators of digit products per slice of columns, one 32-bit integer per lane, four 32-bit "quarter" sums per
(row, bitlayer or pair) in LDS; merged pairs add up in groups that share the accumulators, two 32-bit halves per lane.  This test rebuilds those pieces in exact Python integers for the inputs that make
them largest (every weight digit at its maximum, every activation saturated) at the widest matrix the layout
allows, and checks that each fits the type the kernel gives it and that they recombine to the exact sum.
The limits come from csrc/pb_layout.h (compiled for the host); the digit arithmetic is restated here from
Sections 3.1-3.2 of the paper (plane weights 2^j, the sign plane -2^31; two planes = one base-4 digit).
"""
import ctypes
import itertools
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def limits(tmp_path_factory):
    out = tmp_path_factory.mktemp("limits") / "liblayout_probe.so"
    cmd = ["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-D__host__=", "-D__device__=",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2003_00822_amd", "csrc"),
           "-o", str(out), os.path.join(ROOT, "tests", "layout_probe.cpp")]
    subprocess.check_call(cmd)
    L = ctypes.CDLL(str(out))
    v = (ctypes.c_int * 4)()
    L.probe_limits(v)
    return {"cols": v[0], "cols_pairs": v[1], "slices": v[2], "pair_group": v[3]}


def digits_of(xq):
    """The sixteen base-4 digits of a 32-bit two's-complement value, the top one signed (-2 b31 + b30)."""
    u = xq & 0xFFFFFFFF
    d = [(u >> (2 * i)) & 3 for i in range(16)]
    d[15] = -2 * (d[15] >> 1) + (d[15] & 1)
    assert sum(4 ** i * d[i] for i in range(16)) == (u - (1 << 32) if u >> 31 else u)
    return d


# the four registers of a lane of the result hold the digits b, b + 2, b + 4, b + 6: the quarters
QUARTER_FIRST_DIGIT = [0, 8, 1, 9]
INT32_MAX, INT32_MIN = 2 ** 31 - 1, -2 ** 31
SATURATED = [INT32_MAX, INT32_MIN, 0xFFFF, -1, 0x55555555, -0x55555556, 0x7FFF0000, 1]


def fits_fp32_exactly(v):
    return abs(v) < 2 ** 24


def fits_int32(v):
    return INT32_MIN <= v <= INT32_MAX


@pytest.mark.parametrize("pairs", [False, True])
def test_partial_sums_fit_at_the_widest_matrix(limits, pairs):
    cols = limits["cols_pairs"] if pairs else limits["cols"]
    assert limits["cols_pairs"] <= limits["cols"]
    slice_cols = limits["cols"] // limits["slices"]        # columns of one wave's slice at the widest matrix
    assert slice_cols == 2048
    # weight digit of every column: 0/1 for a single bitlayer; 2 w_hi + w_lo = 0..3 for a pair; the sign pair enters
    # as 2 (1 - w_0) + w_1 = 0..3 and 2 * sum_c x_q[c] is taken off afterwards.  (The kernel keeps the sums of merged
    # pairs as the two halves of the next test; the single word per lane checked here is the tighter form, which a
    # pair by itself would still fit.)
    wdigits = [1] if not pairs else [1, 2, 3]
    for xq, wd, sign_pair in itertools.product(SATURATED, wdigits, [False, True] if pairs else [False]):
        d = digits_of(xq)
        quarters = []
        for b in QUARTER_FIRST_DIGIT:
            # one lane, one slice: fp32 accumulators of digit products
            acc = [wd * d[b + 2 * c] * slice_cols for c in range(4)]
            assert all(fits_fp32_exactly(a) for a in acc)
            t0, t1 = acc[0] + 16 * acc[1], acc[2] + 16 * acc[3]
            assert fits_fp32_exactly(t0) and fits_fp32_exactly(t1)
            lane = t0 + 256 * t1
            assert fits_int32(lane)
            if sign_pair:
                ones = [d[b + 2 * c] * slice_cols for c in range(4)]      # the product with an operand of digits 1
                sx = ones[0] + 16 * ones[1] + 256 * (ones[2] + 16 * ones[3])
                assert fits_int32(sx) and fits_int32(2 * sx)
                lane -= 2 * sx
                assert fits_int32(lane)
            # the LDS word: all slices (and the four lanes that share a slice's columns) add up to all columns
            q = lane * cols // slice_cols
            assert fits_int32(q), (hex(xq & 0xFFFFFFFF), wd, sign_pair, b, q)
            quarters.append(q)
        total = quarters[0] + 4 * quarters[2] + ((quarters[1] + 4 * quarters[3]) << 16)
        signed = xq if xq < 2 ** 31 else xq - 2 ** 32
        eff = wd - 2 if sign_pair else wd
        assert total == eff * signed * cols
        assert abs(total) < 2 ** 63


@pytest.mark.parametrize("last_is_single", [False, True])
def test_group_sums_fit_at_the_widest_matrix(limits, last_is_single):
    """Merged pairs whose scales halve throughout share one set of accumulators: pair p of a group enters with the
    factor 2^e, e = the distance between its low bitlayer and the group's last one (the block scale of the weight
    operand).  Largest case: a full group, every weight digit 3, activations saturated; with an odd bits_used the
    last unit of the last group is a single bitlayer (digit 0/1, factor 1, the pairs before it 2, 8, 32, ...)."""
    cols, G = limits["cols_pairs"], limits["pair_group"]
    slice_cols = limits["cols"] // limits["slices"]
    if last_is_single:
        factors = [2 ** (2 * (G - 1 - p) - 1) for p in range(G - 1)] + [1]
        wdig = [3] * (G - 1) + [1]
    else:
        factors = [4 ** (G - 1 - p) for p in range(G)]
        wdig = [3] * G
    for xq, with_sign_pair in itertools.product(SATURATED, [False, True]):
        d = digits_of(xq)
        halves = []
        for b in QUARTER_FIRST_DIGIT:
            acc = [sum(f * w for f, w in zip(factors, wdig)) * d[b + 2 * c] * slice_cols for c in range(4)]
            assert all(fits_fp32_exactly(a) for a in acc), (hex(xq & 0xFFFFFFFF), acc)
            i0, i1 = acc[0] + 16 * acc[1], acc[2] + 16 * acc[3]       # converted register by register, as integers
            assert fits_int32(i0) and fits_int32(i1)
            w0, w1 = i0 * cols // slice_cols, i1 * cols // slice_cols      # the LDS words: all slices of a row
            assert fits_int32(w0) and fits_int32(w1), (hex(xq & 0xFFFFFFFF), b, w0, w1)
            if with_sign_pair:
                # pair 0 of the group is the sign pair: 2 * sum_c x_q[c] times its factor is what its digits count too
                # much; the slices add their shares up in LDS words of the same form, once per call, and the final sum
                # takes them off the row's words
                ones = [d[b + 2 * c] * slice_cols for c in range(4)]
                s0, s1 = (ones[0] + 16 * ones[1]) * 2 * factors[0], (ones[2] + 16 * ones[3]) * 2 * factors[0]
                assert fits_int32(s0) and fits_int32(s1)                       # a slice's share
                s0, s1 = s0 * cols // slice_cols, s1 * cols // slice_cols
                assert fits_int32(s0) and fits_int32(s1), (hex(xq & 0xFFFFFFFF), b, s0, s1)
                w0, w1 = w0 - s0, w1 - s1
                assert fits_int32(w0) and fits_int32(w1)
            halves.append(w0 + 256 * w1)
        total = halves[0] + 4 * halves[2] + ((halves[1] + 4 * halves[3]) << 16)
        signed = xq if xq < 2 ** 31 else xq - 2 ** 32
        eff = [w - 2 if (with_sign_pair and p == 0) else w for p, w in enumerate(wdig)]
        assert total == sum(f * e for f, e in zip(factors, eff)) * signed * cols
        assert abs(total) < 2 ** 63


def test_popcount_kernel_halves_fit(limits):
    """The AND + popcount kernel keeps sum_j 2^j P_j of the planes 0-15 and 16-31 apart as two 32-bit integers:
    at 32768 columns the low half reaches 32768 * 65535 < 2^31 and the high half -32768 * 32768 = -2^30."""
    cols = 32768
    lo_max = cols * 0xFFFF
    hi_min, hi_max = cols * -(1 << 15), cols * 0x7FFF
    assert fits_int32(lo_max) and fits_int32(hi_min) and fits_int32(hi_max)
    assert lo_max + (hi_min << 16) == cols * ((INT32_MIN) + 0xFFFF)
