"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Integer accumulators and codes bit-exact; fp32 outputs within 1e-5 relative."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import pb_oracle as po
from paper_2003_00822_amd import synth
from tests.helpers import assert_y_close, oracle_reference, pair_sums

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pb():
    assert torch.cuda.is_available(), "gpu tests need a GPU"
    from paper_2003_00822_amd import pb as pbmod
    pbmod.lib()  # fails loudly if the HIP library is missing
    return pbmod


# every case runs on the packed layouts: the matrix-core kernel (default), the AND + popcount kernel, and the
# matrix-core kernel on the layout that stores the digits of the bitlayer pairs
LAYOUTS = {"mfma": 0x50420002, "popc": 0x50420001, "pair": 0x50420004}


@pytest.fixture(params=sorted(LAYOUTS), scope="module")
def layout(request):
    return LAYOUTS[request.param]


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_layer(pb, W, bits, X, m_list, frac_bits=16, act_bits=32, check_y=True, layout=None):
    R, C = W.shape
    N = X.shape[0]
    lin = pb.PackedLinear(dev(W), bits, max_batch=N, frac_bits=frac_bits, act_bits=act_bits, layout=layout)
    assert layout is None or lin.desc.layout == layout
    prep = po.prepare(W, bits)
    # Algorithm 1: codes and scales
    q_gpu = lin.unpack().cpu().numpy()
    assert (q_gpu == prep["q"]).all(), "quantized codes differ"
    sc_gpu = lin.scales[:bits].cpu().numpy()
    assert (sc_gpu.view(np.int32) == prep["scales"].view(np.int32)).all(), "scales differ"
    Xd = dev(X)
    for m in m_list:
        ref = oracle_reference(W, bits, X, m, frac_bits=frac_bits, act_bits=act_bits)
        A_gpu = lin.acc(Xd, m).cpu().numpy()
        assert A_gpu.shape == ref["A"].shape
        bad = A_gpu != ref["A"]
        assert not bad.any(), "int64 accumulators differ at %s (R=%d C=%d bits=%d m=%d)" % (
            np.argwhere(bad)[:5].tolist(), R, C, bits, m)
        if lin.desc.layout != LAYOUTS["popc"]:
            # the sums of the bitlayer pairs, as the matrix-core kernel holds them on its usual route
            P_gpu = lin.acc_pairs(Xd, m).cpu().numpy()
            bad = P_gpu != pair_sums(ref["A"], m)
            assert not bad.any(), "pair sums differ at %s (R=%d C=%d bits=%d m=%d)" % (
                np.argwhere(bad)[:5].tolist(), R, C, bits, m)
        if check_y:
            Y_gpu = lin(Xd, m).cpu().numpy()
            assert_y_close(Y_gpu, ref["Y"], ref["A"], prep["scales"], frac_bits=frac_bits)
    return lin


SHAPES = [
    (1, 1), (3, 5), (4, 32), (5, 33), (7, 64), (16, 127), (33, 128), (10, 4096), (64, 96), (130, 784),
    (257, 1024), (100, 3000), (33, 4100), (17, 8192 + 5), (9, 16384), (4100, 40), (6, 12000), (9, 16385),
    (18, 20000), (5, 32768),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_shapes_all_layers(pb, layout, shape):
    R, C = shape
    bits = 1 + (R + C) % 8
    W, X = synth.ragged(R, C, batch=1, case=1)
    print("shape", shape, "bits", bits, flush=True)
    run_layer(pb, W, bits, X, sorted({1, bits, max(1, bits // 2)}), layout=layout)


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 5, 6, 7, 8, 12, 16])
def test_every_bit_width_and_prefix(pb, layout, bits):
    W, X = synth.ragged(70, 200, batch=1, case=bits, xdist="uniform")
    print("bits", bits, flush=True)
    run_layer(pb, W, bits, X, list(range(1, bits + 1)), layout=layout)


TILED = ["mfma", "pair"]    # the two layouts of the matrix-core kernel


@pytest.mark.parametrize("lay", TILED)
@pytest.mark.parametrize("bits", [2, 3, 5, 8])
def test_scales_that_do_not_halve_are_applied_bitlayer_by_bitlayer(pb, bits, lay):
    """Any fp32 scales are legal input: the kernel merges bitlayer pairs only if scales[i] == 2 scales[i+1] throughout."""
    W, X = synth.ragged(50, 1500, batch=3, case=40 + bits, xdist="normal")
    lin = pb.PackedLinear(dev(W), bits, max_batch=3, layout=LAYOUTS[lay])
    ref = oracle_reference(W, bits, X, bits)
    rng = np.random.default_rng(bits)
    for kind in ("random", "one_off"):
        sc = ref["scales"].copy()
        if kind == "random":
            sc = (sc * rng.uniform(0.5, 1.5, size=bits)).astype(np.float32)
        else:
            sc[-1] = np.nextafter(sc[-1], np.float32(1.0))   # a single ulp breaks the ratio of the last pair
        lin.scales[:bits] = dev(sc)
        Y = np.zeros((3, 50))
        for i in range(bits):
            Y += float(sc[i]) * ref["A"][i].astype(np.float64)
        Y_ref = (Y * 2.0 ** -16).astype(np.float32)
        print("bits", bits, kind, flush=True)
        assert_y_close(lin(dev(X), bits).cpu().numpy(), Y_ref, ref["A"], sc)


@pytest.mark.parametrize("lay", TILED)
@pytest.mark.parametrize("bits", [9, 10, 11, 12, 16])
def test_pair_groups_share_accumulators(pb, bits, lay):
    """Batches with scales that halve throughout: up to five bitlayer pairs of a row tile add up in one set of
    registers (pair p with the factor 4^(last - p), supplied by the block scale of the weight operand), further
    pairs in a second group; prefixes on both sides of the group boundaries, with and without a last single bitlayer."""
    for (R, C, N, case) in ((40, 1300, 3, 81), (17, 9000, 5, 82)):
        W, X = synth.ragged(R, C, batch=N, case=case + bits, xdist="wide")
        ms = sorted(m for m in {1, 2, 3, 9, 10, 11, 12, bits - 1, bits} if 1 <= m <= bits)
        print("pair groups", bits, R, C, N, ms, flush=True)
        run_layer(pb, W, bits, X, ms, layout=LAYOUTS[lay])


@pytest.mark.parametrize("lay", TILED)
@pytest.mark.parametrize("bits", [10, 11, 16])
def test_pair_groups_at_their_limits(pb, bits, lay):
    """A full group of five pairs (and five pairs plus more) at 32768 columns, every weight digit at its maximum,
    activations saturated: the shared accumulators and the 32-bit halves in LDS are as large as they get
    (tests/test_accumulator_bounds.py works the bounds out on the host)."""
    cols = 32768
    X = limit_vectors(cols)
    for name, W in limit_matrices(cols, bits):
        print("pair groups at the limits", bits, name, flush=True)
        run_layer(pb, W, bits, X, [9, 10, bits], layout=LAYOUTS[lay])
        run_layer(pb, W, bits, X[:2], [10], layout=LAYOUTS[lay])


@pytest.mark.parametrize("xdist", ["normal", "uniform", "relu", "wide"])
def test_activation_distributions(pb, layout, xdist):
    W, X = synth.ragged(96, 1000, batch=3, case=3, xdist=xdist)
    print("xdist", xdist, flush=True)
    run_layer(pb, W, 4, X, [1, 4], layout=layout)


@pytest.mark.parametrize("shape_batch", [(40, 700, 5), (33, 4096, 7), (20, 5000, 3), (18, 8192, 6), (17, 9000, 2), (20, 17000, 3),
                                         (25, 3000, 20), (19, 4096, 17), (21, 2000, 26)])
def test_batches_that_do_not_fill_a_vector_group(pb, layout, shape_batch):
    R, C, N = shape_batch
    W, X = synth.ragged(R, C, batch=N, case=11, xdist="normal")
    print("batch", shape_batch, flush=True)
    run_layer(pb, W, 3, X, [1, 3], layout=layout)


def test_maximum_batch(pb, layout):
    """PB_MAX_BATCH vectors in one call (many vector groups per row tile; the last group is full)."""
    W, X = synth.ragged(20, 600, batch=pb.PB_MAX_BATCH, case=12, xdist="normal")
    print("batch", pb.PB_MAX_BATCH, flush=True)
    run_layer(pb, W, 3, X, [3], layout=layout)
    # one vector short of a full last group
    run_layer(pb, W, 4, X[: pb.PB_MAX_BATCH - 1], [2], layout=layout)


def test_random_configurations(pb):
    """Seeded random shapes, widths, prefixes, batches, activation formats and distributions on the layouts of the
    matrix-core kernel: codes, per-bitlayer sums, pair sums and outputs against the oracle."""
    rng = np.random.default_rng(200300822)
    for case in range(120):
        R = int(rng.integers(1, 160))
        C = int(rng.choice([rng.integers(1, 700), rng.integers(700, 4200), rng.integers(4200, 9000)]))
        N = int(rng.choice([1, 1, 2, 3, 5, 8, 9, 17]))
        bits = int(rng.integers(1, 17))
        m = sorted({int(rng.integers(1, bits + 1)), bits})
        act_bits, frac_bits = [(32, 16), (32, 16), (16, 12), (8, 4), (24, 20)][int(rng.integers(0, 5))]
        xdist = ["normal", "uniform", "relu", "wide"][int(rng.integers(0, 4))]
        W, X = synth.ragged(R, C, batch=N, case=100 + case, xdist=xdist)
        print("case", case, (R, C, N), "bits", bits, "m", m, "act", act_bits, frac_bits, xdist, flush=True)
        lay = GATES if (R % 4 == 0 and case % 3 == 0) else LAYOUTS["mfma" if case % 2 else "pair"]
        run_layer(pb, W, bits, X, m, frac_bits=frac_bits, act_bits=act_bits, layout=lay)


def test_random_configurations_of_the_multi_pass_kernels(pb):
    """Seeded random widths and batches on both sides of every threshold at which the launcher takes the columns in
    several passes (rows beyond 4096 columns with 33 and more operands on the bit layout, beyond 8192 columns from a
    few operands on, four or eight operands per wave), with ragged last passes and groups that are not full."""
    rng = np.random.default_rng(200300822 + 7)
    for case in range(96):
        R = int(rng.integers(1, 48))
        if case % 2:
            C = int(rng.integers(4097, 8193))
            N = int(rng.choice([31, 32, 33, 36, 37, 40, 45, 64, 70]))
        else:
            C = int(rng.choice([rng.integers(8193, 12289), rng.integers(12289, 16385), rng.integers(16385, 32769)]))
            N = int(rng.choice([2, 3, 4, 5, 8, 12, 16, 17, 21, 24, 25, 40]))
        bits = int(rng.integers(1, 11))
        m = sorted({int(rng.integers(1, bits + 1)), bits})
        act_bits, frac_bits = [(32, 16), (32, 16), (16, 12), (8, 4)][int(rng.integers(0, 4))]
        W, X = synth.ragged(R, C, batch=N, case=400 + case, xdist=["normal", "wide"][case % 3 == 0])
        lay = GATES if (R % 4 == 0 and case % 5 == 0) else LAYOUTS["pair" if case % 4 >= 2 else "mfma"]
        print("case", case, (R, C, N), "bits", bits, "m", m, "act", act_bits, frac_bits, hex(lay), flush=True)
        run_layer(pb, W, bits, X, m, frac_bits=frac_bits, act_bits=act_bits, layout=lay)


def test_fixed_point_conversion(pb):
    u = 2.0 ** -16
    special = [0.0, 1.0, -2.0, 0.5 * u, -0.5 * u, 1.5 * u, -1.5 * u, 1.0 - 2.0 ** -24, 32767.998046875, 32768.0,
               -32768.0, -32768.5, 1e30, -1e30, float("inf"), float("-inf"), float("nan"), -0.0]
    rng = np.random.default_rng(4)
    x = np.concatenate([np.array(special, dtype=np.float32),
                        (rng.normal(size=3000) * np.exp2(rng.integers(-30, 18, size=3000))).astype(np.float32)])
    X = x.reshape(1, -1)
    for (f, k) in [(16, 32), (8, 32), (16, 16), (4, 8), (0, 4)]:
        d = pb.pb_desc_init(4, X.shape[1], 2, frac_bits=f, act_bits=k)
        ws = pb.alloc_workspace(d, 1)
        xq = torch.empty(X.shape, dtype=torch.int32, device="cuda")
        pb.pb_fixed_point(d, dev(X), 1, xq, ws)
        want = po.fixed_point(X, frac_bits=f, act_bits=k)
        assert (xq.cpu().numpy() == want).all(), (f, k)


def test_special_activation_vectors(pb, layout):
    R, C, bits = 37, 200, 5
    W, _ = synth.ragged(R, C, case=2)
    cases = {
        "zeros": np.zeros((1, C), dtype=np.float32),
        "minus_one_lsb": np.full((1, C), -1.0 / 65536, dtype=np.float32),   # x_q = -1: every plane all ones
        "int32_min": np.full((1, C), -40000.0, dtype=np.float32),           # only the negative top plane
        "int32_max": np.full((1, C), 40000.0, dtype=np.float32),
        "tiny": np.full((1, C), 1.0 / 65536, dtype=np.float32),             # x_q = 1: one plane
    }
    onehot = np.zeros((1, C), dtype=np.float32)
    onehot[0, 131] = -3.25
    cases["onehot"] = onehot
    for name, X in cases.items():
        print("special", name, flush=True)
        run_layer(pb, W, bits, X, [1, 3, 5], layout=layout)


def test_non_finite_and_signed_zero_activations(pb, layout):
    """NaN converts to 0, +-inf saturate, -0.0 is 0 (Algorithm 2's Int(x * 2^16) as the interface defines it for
    values a cast does not cover), through the conversion inside the product kernels: batch 1, batches that
    fill and that do not fill a vector group, a vector of nothing but NaN, one of -inf."""
    R, C, bits = 45, 1300, 5
    W, X = synth.ragged(R, C, batch=9, case=41, xdist="normal")
    X = X.copy()
    rng = np.random.default_rng(200300822 + 41)
    idx = rng.choice(X.size, size=X.size // 6, replace=False)
    X.flat[idx] = rng.choice(np.array([np.nan, np.inf, -np.inf, -0.0, 0.0, 3.0e38, -3.0e38, 1e-40, -1e-40],
                                      dtype=np.float32), size=idx.size)
    X[3, :] = np.nan
    X[4, :] = -np.inf
    X[:, 517] = np.inf          # a whole column
    X[:, 1299] = np.nan         # the last one
    for N in (1, 2, 5, 9):
        print("non-finite, batch", N, flush=True)
        run_layer(pb, W, bits, X[:N], [1, 4, 5], layout=layout)
    # narrower activations: +-inf saturate at the k-bit range
    run_layer(pb, W, bits, X[:5], [5], frac_bits=4, act_bits=8, layout=layout)


def test_non_finite_activations_in_a_concatenated_input(pb):
    """The LSTM wrapper's [x_t ; h] input: both parts go through the same conversion."""
    H, I, bits, N = 37, 100, 4, 3
    g = np.random.default_rng(200300822 + 43)
    W = g.uniform(-0.04, 0.04, size=(4 * H, I + H)).astype(np.float32)
    x = g.normal(size=(N, I)).astype(np.float32)
    h = g.uniform(-1, 1, size=(N, H)).astype(np.float32)
    c = g.uniform(-1, 1, size=(N, H)).astype(np.float32)
    x[0, 5] = np.nan; x[1, 99] = np.inf; h[2, 0] = -np.inf; h[0, 36] = np.nan; x[2, 0] = -0.0
    for lay in (GATES, LAYOUTS["mfma"]):
        lin = pb.PackedLinear(dev(W), bits, max_batch=N, layout=lay)
        prep = po.prepare(W, bits)
        lw = po.pack_words(prep["layers"])
        xh = np.concatenate([x, h], axis=1)
        _, Y = po.matmul_words(lw, prep["scales"], bits, I + H, xh)
        h_ref, c_ref = po.lstm_pointwise(Y, None, c)
        h_out = torch.empty((N, H), dtype=torch.float32, device="cuda")
        c_out = torch.empty((N, H), dtype=torch.float32, device="cuda")
        pb.pb_lstm_cell(lin.packed, lin.scales, lin.desc, bits, dev(x), I, dev(h), dev(c), None, h_out, c_out, N,
                        lin.workspace)
        assert np.abs(h_out.cpu().numpy() - h_ref).max() <= 2e-6
        assert np.abs(c_out.cpu().numpy() - c_ref).max() <= 2e-6


def limit_matrices(cols, bits):
    """Weight codes that put every partial sum of the kernels at its bound: all -1 (every bitlayer all ones; a row
    of its own holds +qmax, which fixes the step at 1) and all +qmax (sign bitlayer empty, all others full: the
    largest digit of every bitlayer pair, the sign pair included)."""
    qmax = 2 ** (bits - 1) - 1
    Wa = -np.ones((18, cols), dtype=np.float32)
    Wa[17, :] = 0.0
    Wa[17, 0] = float(qmax)
    Wb = np.full((17, cols), float(qmax), dtype=np.float32)
    return [("all ones", Wa), ("all qmax", Wb)]


def limit_vectors(cols):
    """Saturated activations: x_q = INT32_MAX, INT32_MIN, 0xFFFF, -1, alternating extremes."""
    X = np.empty((5, cols), dtype=np.float32)
    X[0] = 40000.0
    X[1] = -40000.0
    X[2] = 65535.0 / 65536.0
    X[3] = -1.0 / 65536.0
    X[4] = np.where(np.arange(cols) % 2 == 0, 40000.0, -40000.0)
    return X


@pytest.mark.parametrize("cols", [32768, 16384, 32768 - 31])
def test_partial_sums_at_their_limits(pb, layout, cols):
    """The widest matrices times saturated activations: the 32-bit pieces in which the kernels hold the exact sums of
    Algorithm 2 are as large as they get (tests/test_accumulator_bounds.py works the bounds out on the host).
    Single bitlayers, bitlayer pairs (sign pair included), batch 1 and a batch."""
    bits = 8
    X = limit_vectors(cols)
    for name, W in limit_matrices(cols, bits):
        prep = po.prepare(W, bits)
        assert prep["d"] == 1.0 and int(prep["q"].min()) in (-1, 2 ** (bits - 1) - 1)
        print("limits", cols, name, "batch 5", flush=True)
        run_layer(pb, W, bits, X, [1, 2, 7, 8], layout=layout)
        for n in range(5):
            print("limits", cols, name, "vector", n, flush=True)
            run_layer(pb, W, bits, X[n:n + 1], [2, 8], layout=layout)


@pytest.mark.parametrize("lay", TILED)
@pytest.mark.parametrize("fk", [(2, 4), (4, 8), (5, 9), (12, 16), (7, 12)])
def test_vectors_that_share_an_operand(pb, fk, lay):
    """Activations of at most 16 (8) bits: two (four) vectors travel in one operand of the matrix-core kernel.
    Batches that fill the operands and that leave sub-vectors or whole operands empty, every route (per-bitlayer
    sums, pair sums, fp32 output), inputs that saturate at k bits."""
    f, k = fk
    for (R, C, N, case) in ((45, 1300, 2, 71), (33, 520, 3, 72), (20, 4200, 4, 73), (50, 300, 5, 74),
                            (17, 9000, 9, 75), (40, 2100, 17, 76), (18, 700, 33, 77)):
        print("shared operands", fk, R, C, N, flush=True)
        W, X = synth.ragged(R, C, batch=N, case=case, xdist="wide" if case % 2 else "uniform")
        run_layer(pb, W, 5, X, [1, 2, 5], frac_bits=f, act_bits=k, layout=LAYOUTS[lay])


@pytest.mark.parametrize("lay", TILED)
@pytest.mark.parametrize("k", [8, 16])
def test_shared_operands_at_their_limits(pb, k, lay):
    """All-ones / all-qmax bitlayers times activations saturated at k bits, 32768 columns, batches of 4 and 5."""
    cols, bits = 32768, 8
    X = limit_vectors(cols)                     # +-40000 saturate at +-2^(k-1) with frac_bits = k - 2
    for name, W in limit_matrices(cols, bits):
        print("shared operands at the limits", k, name, flush=True)
        run_layer(pb, W, bits, X, [2, 7, 8], frac_bits=k - 2, act_bits=k, layout=LAYOUTS[lay])
        run_layer(pb, W, bits, X[:4], [8], frac_bits=k - 2, act_bits=k, layout=LAYOUTS[lay])


def test_lstm_cell_with_narrow_activations_and_batch(pb):
    """The fused cell update on operands that several vectors share (act_bits = 8, batch 6)."""
    H, I, bits, N = 37, 100, 4, 6
    g = np.random.default_rng(200300822 + 47)
    W = g.uniform(-0.04, 0.04, size=(4 * H, I + H)).astype(np.float32)
    x = g.normal(size=(N, I)).astype(np.float32)
    h = g.uniform(-1, 1, size=(N, H)).astype(np.float32)
    c = g.uniform(-1, 1, size=(N, H)).astype(np.float32)
    bias = g.normal(0, 0.1, size=4 * H).astype(np.float32)
    prep = po.prepare(W, bits)
    lw = po.pack_words(prep["layers"])
    xh = np.concatenate([x, h], axis=1)
    _, Y = po.matmul_words(lw, prep["scales"], bits, I + H, xh, frac_bits=5, act_bits=8)
    h_ref, c_ref = po.lstm_pointwise(Y, bias, c)
    for lay in (GATES, LAYOUTS["mfma"]):
        lin = pb.PackedLinear(dev(W), bits, max_batch=N, frac_bits=5, act_bits=8, layout=lay)
        h_out = torch.empty((N, H), dtype=torch.float32, device="cuda")
        c_out = torch.empty((N, H), dtype=torch.float32, device="cuda")
        pb.pb_lstm_cell(lin.packed, lin.scales, lin.desc, bits, dev(x), I, dev(h), dev(c), dev(bias), h_out, c_out, N,
                        lin.workspace)
        assert np.abs(h_out.cpu().numpy() - h_ref).max() <= 2e-6
        assert np.abs(c_out.cpu().numpy() - c_ref).max() <= 2e-6


def test_reduced_activation_precision(pb, layout):
    # Section 3.1: k (activation precision) of 8 or 16 planes; the fixed point moves with it
    W, X = synth.ragged(50, 300, batch=2, case=5, xdist="uniform")
    for (f, k) in [(6, 8), (14, 16), (20, 32)]:
        print("act", f, k, flush=True)
        run_layer(pb, W, 4, X, [2, 4], frac_bits=f, act_bits=k, layout=layout)


@pytest.mark.parametrize("fmt", [(32, 16, 2, "normal"), (8, 4, 1, "wide"), (16, 12, 5, "wide"), (32, 16, 9, "wide")])
def test_prepared_halves_equal_whole_call(pb, layout, fmt):
    """pb_act_prep + pb_matmul_prepared (planes through memory) against pb_matmul and the oracle."""
    act_bits, frac_bits, N, xdist = fmt
    W, X = synth.ragged(150, 2100, batch=N, case=7, xdist=xdist)
    bits, m = 6, 5
    lin = pb.PackedLinear(dev(W), bits, max_batch=N, layout=layout, frac_bits=frac_bits, act_bits=act_bits)
    ref = oracle_reference(W, bits, X, m, frac_bits=frac_bits, act_bits=act_bits)
    Xd = dev(X)
    Y1 = lin(Xd, m).cpu().numpy()
    Y2 = torch.empty((N, 150), dtype=torch.float32, device="cuda")
    pb.pb_act_prep(lin.desc, Xd, N, lin.workspace)
    pb.pb_matmul_prepared(lin.packed, lin.scales, lin.desc, m, N, Y2, lin.workspace)
    assert_y_close(Y1, ref["Y"], ref["A"], ref["scales"], frac_bits=frac_bits)
    assert (Y2.cpu().numpy().view(np.int32) == Y1.view(np.int32)).all()


@pytest.mark.parametrize("lay", TILED)
@pytest.mark.parametrize("shape_batch", [(60, 9000, 9), (33, 20000, 6), (40, 6000, 40)])
def test_prepared_planes_on_the_multi_pass_kernels(pb, lay, shape_batch):
    """Bit planes handed over in memory (pb_act_prep + pb_matmul_prepared) on rows and batches that the matrix-core
    kernel takes in several passes over the columns: same bits as the call that converts the activations itself."""
    R, C, N = shape_batch
    W, X = synth.ragged(R, C, batch=N, case=31, xdist="wide")
    bits, m = 6, 5
    lin = pb.PackedLinear(dev(W), bits, max_batch=N, layout=LAYOUTS[lay])
    ref = oracle_reference(W, bits, X, m)
    Xd = dev(X)
    Y1 = lin(Xd, m).cpu().numpy()
    Y2 = torch.empty((N, R), dtype=torch.float32, device="cuda")
    pb.pb_act_prep(lin.desc, Xd, N, lin.workspace)
    pb.pb_matmul_prepared(lin.packed, lin.scales, lin.desc, m, N, Y2, lin.workspace)
    assert_y_close(Y1, ref["Y"], ref["A"], ref["scales"])
    assert (Y2.cpu().numpy().view(np.int32) == Y1.view(np.int32)).all()


@pytest.mark.parametrize("fk", [(6, 8), (10, 16), (14, 16)])
def test_narrow_activations_with_batch_and_saturation(pb, fk):
    """act_bits <= 16 (Section 3.1: fewer activation bits) on the matrix-core kernel; wide inputs saturate at k bits."""
    f, k = fk
    W, X = synth.ragged(90, 1300, batch=5, case=23, xdist="wide")
    run_layer(pb, W, 6, X, [1, 4, 6], frac_bits=f, act_bits=k, layout=LAYOUTS["mfma"])
    W, X = synth.ragged(40, 5000, batch=1, case=29, xdist="normal")
    run_layer(pb, W, 3, X, [3], frac_bits=f, act_bits=k, layout=LAYOUTS["mfma"])


def test_config1_fc_1024_definition_level(pb, layout):
    """Config 1, checked against the byte-per-bit tier of the oracle (Algorithm 2 taken literally)."""
    W, X = synth.fc_small()
    bits = 4
    prep = po.prepare(W, bits)
    lin = pb.PackedLinear(dev(W), bits, layout=layout)
    for m in range(1, bits + 1):
        A, T, Y = po.matmul_bitserial(prep["layers"], prep["scales"], prep["s"], m, X)
        A_gpu = lin.acc(dev(X), m).cpu().numpy()
        assert (A_gpu == A).all()
        Y_gpu = lin(dev(X), m).cpu().numpy()
        assert_y_close(Y_gpu, Y, A, prep["scales"])


@pytest.mark.parametrize("bits", [8, 3])
def test_config2_fc_4096_full_size(pb, layout, bits):
    W, X = synth.fc_square(4096, 0.02)
    print("cfg2 bits", bits, flush=True)
    run_layer(pb, W, bits, X, list(range(1, bits + 1)), layout=layout)


def test_config3_mlp_layers(pb, layout):
    """Config 3: each layer fed with the oracle's previous-layer output (ReLU), so integers must match."""
    Ws, X = synth.mlp()
    bits = 6
    x = X
    for li, W in enumerate(Ws):
        print("mlp layer", li, W.shape, flush=True)
        m = [bits, 2, 4][li]
        run_layer(pb, W, bits, x, [m], layout=layout)
        ref = oracle_reference(W, bits, x, m)
        x = np.maximum(ref["Y"], 0.0).astype(np.float32)


def test_config5_large_fc_batch(pb, layout):
    W, X = synth.fc_large(batch=4)
    print("cfg5 8192 batch 4", flush=True)
    run_layer(pb, W, 2, X, [2], layout=layout)
    W16, X16 = synth.ragged(64, 8192, batch=16, case=9)
    run_layer(pb, W16, 8, X16, [8], layout=layout)


def test_config5_full_size_batch_64_sampled_rows(pb, layout):
    """Config 5 at its largest: 8192 x 8192, B = 8, batch 64, in the launch configuration the benchmark times;
    the oracle computes sampled rows (all 64 vectors, all bitlayers) one by one."""
    W, X = synth.fc_large(batch=64)
    bits = 8
    lin = pb.PackedLinear(dev(W), bits, max_batch=64, layout=layout)
    rng = np.random.default_rng(5)
    rows = sorted(set(rng.choice(8192, size=20, replace=False).tolist() + [0, 15, 16, 8191]))
    Xd = dev(X)
    A_gpu = lin.acc(Xd, bits).cpu().numpy()
    Y_gpu = lin(Xd, bits).cpu().numpy()
    prep = po.prepare(W, bits)
    xq = po.fixed_point(X)
    for r in rows:
        sub = po.layer_products_direct(prep["layers"][:, r:r + 1, :], bits, xq)      # [bits, 64, 1]
        assert (A_gpu[:, :, r] == sub[:, :, 0]).all(), r
        y = po.dequant(sub[:, :, 0], prep["scales"], bits)
        assert_y_close(Y_gpu[:, r], y, sub[:, :, 0], prep["scales"])


@pytest.mark.parametrize("bits", [1, 2, 5, 8])
def test_pairs_layout_words(pb, bits):
    """The stored words of PB_LAYOUT_TILE16_PAIRS_V1 against its definition, worked out in numpy from the words of the
    default layout (same blocks, same positions): digit d_c = 2 upper_c + lower_c of the bitlayers (2p, 2p + 1), even
    columns of a word in the block of bitlayer 2p (two bits at c), odd columns in the block of bitlayer 2p + 1 (two
    bits at c - 1); bitlayer 0 complemented; a last single bitlayer paired with zeros."""
    W, _ = synth.ragged(37, 1100, batch=1, case=300 + bits)
    plain = pb.PackedLinear(dev(W), bits)
    pairs = pb.PackedLinear(dev(W), bits, layout=LAYOUTS["pair"])
    stored = (bits + 1) & ~1
    a = plain.packed.cpu().numpy().view(np.uint32).reshape(bits, -1)
    b = pairs.packed.cpu().numpy().view(np.uint32).reshape(stored, -1)
    assert pairs.packed.numel() == stored * a.shape[1] * 4
    for p in range(stored // 2):
        upper = a[2 * p].copy()
        if p == 0:
            upper = ~upper
        lower = a[2 * p + 1] if 2 * p + 1 < bits else np.zeros_like(upper)
        even = (lower & np.uint32(0x55555555)) | ((upper << np.uint32(1)) & np.uint32(0xAAAAAAAA))
        odd = ((lower >> np.uint32(1)) & np.uint32(0x55555555)) | (upper & np.uint32(0xAAAAAAAA))
        assert (b[2 * p] == even).all(), (bits, p, "even columns")
        assert (b[2 * p + 1] == odd).all(), (bits, p, "odd columns")


@pytest.mark.parametrize("lay", TILED)
def test_repeated_full_size_calls_are_bit_identical(pb, lay):
    """All integer sums are exact, so a call's output does not depend on the schedule of its waves: the same call
    repeated on the full grid (8192 x 8192, the launch configurations the benchmark times: one vector, a few
    vectors, batch 64, and four vectors per operand) gives the same bits every time, whatever ran before it."""
    torch.manual_seed(77)
    n = 8192
    W = torch.randn((n, n), device="cuda") * 0.01
    X = torch.randn((64, n), device="cuda")
    for (bits, act_bits, frac_bits) in ((8, 32, 16), (5, 8, 4)):
        lin = pb.PackedLinear(W, bits, max_batch=64, frac_bits=frac_bits, act_bits=act_bits, layout=LAYOUTS[lay])
        for N, m in ((1, bits), (1, 3), (5, bits), (64, bits), (64, bits - 1)):
            first = lin(X[:N], m).clone()
            for rep in range(6):
                lin(X[(rep % 3):(rep % 3) + 1], 1 + rep % bits)      # other work in between
                again = lin(X[:N], m)
                assert torch.equal(first, again), (lay, bits, act_bits, N, m, rep)


def test_extra_16384(pb, layout):
    W, X = synth.fc_square(16384, 0.01, cfg=6)
    bits = 2
    lin = pb.PackedLinear(dev(W), bits, layout=layout)
    # oracle on sampled rows only (full size in the launch configuration of the benchmark)
    rng = np.random.default_rng(0)
    rows = sorted(rng.choice(16384, size=48, replace=False).tolist() + [0, 16383])
    A_gpu = lin.acc(dev(X), bits).cpu().numpy()
    Y_gpu = lin(dev(X), bits).cpu().numpy()
    prep = po.prepare(W, bits)
    xq = po.fixed_point(X)
    for r in rows:
        sub = po.layer_products_direct(prep["layers"][:, r:r + 1, :], bits, xq)
        assert (A_gpu[:, :, r] == sub[:, :, 0]).all(), r
        y = po.dequant(sub[:, 0, :], prep["scales"], bits)
        assert_y_close(Y_gpu[:, r], y, sub[:, 0, :], prep["scales"])


@pytest.mark.parametrize("lay", TILED)
def test_wide_rows_in_several_passes(pb, lay):
    """Batches on rows of more than 8192 columns: the kernel covers the columns in several passes over the same row
    tiles (16500 columns: five passes of eight operands per wave, or three of four operands where four vectors share
    an operand), whose sums wait in LDS for the last pass, as many row tiles at a time as have room: 207 row tiles
    on a few workgroups per vector group make every workgroup go through several such rounds, with every kind of
    sums (groups of pairs, pair by pair, bitlayer by bitlayer with scales that do not halve) and one, two and four
    vectors per operand.  The oracle computes sampled rows."""
    R, C, N, bits = 3300, 16500, 256, 8
    W, X = synth.ragged(R, C, batch=N, case=91, xdist="normal")
    rng = np.random.default_rng(91)
    rows = sorted(set(rng.choice(R, size=12, replace=False).tolist() + [0, 15, 16, R - 1]))
    prep = po.prepare(W, bits)
    Xd = dev(X)
    for (act_bits, frac_bits, m) in ((32, 16, 8), (32, 16, 5), (16, 10, 7), (8, 4, 8)):
        print("wide rows", lay, act_bits, m, flush=True)
        lin = pb.PackedLinear(dev(W), bits, max_batch=N, frac_bits=frac_bits, act_bits=act_bits, layout=LAYOUTS[lay])
        Y_gpu = lin(Xd, m).cpu().numpy()
        P_gpu = lin.acc_pairs(Xd, m).cpu().numpy()
        sc = prep["scales"].copy()
        sc[1] = np.nextafter(sc[1], np.float32(1.0))       # one ulp: no pair is merged
        lin.scales[:bits] = dev(sc)
        Y2_gpu = lin(Xd, m).cpu().numpy()
        xq = po.fixed_point(X, frac_bits=frac_bits, act_bits=act_bits)
        for r in rows:
            sub = po.layer_products_direct(prep["layers"][:, r:r + 1, :], m, xq)[:, :, 0]      # [m, N]
            assert (P_gpu[:, :, r] == pair_sums(sub[:, :, None], m)[:, :, 0]).all(), (r, "pair sums")
            y = po.dequant(sub, prep["scales"], m, frac_bits=frac_bits)
            assert_y_close(Y_gpu[:, r], y, sub, prep["scales"], frac_bits=frac_bits)
            y2 = np.zeros(N)
            for i in range(m):
                y2 += float(sc[i]) * sub[i].astype(np.float64)
            assert_y_close(Y2_gpu[:, r], (y2 * 2.0 ** -frac_bits).astype(np.float32), sub, sc, frac_bits=frac_bits)


def test_wide_rows_lstm_cell_with_batch(pb):
    """The fused cell update at the end of the last of two passes over the columns (8440 columns, batch 5)."""
    H, I, bits, N = 40, 8400, 4, 5
    g = np.random.default_rng(200300822 + 53)
    W = g.uniform(-0.01, 0.01, size=(4 * H, I + H)).astype(np.float32)
    x = g.normal(size=(N, I)).astype(np.float32)
    h = g.uniform(-1, 1, size=(N, H)).astype(np.float32)
    c = g.uniform(-1, 1, size=(N, H)).astype(np.float32)
    bias = g.normal(0, 0.1, size=4 * H).astype(np.float32)
    prep = po.prepare(W, bits)
    lw = po.pack_words(prep["layers"])
    xh = np.concatenate([x, h], axis=1)
    _, Y = po.matmul_words(lw, prep["scales"], bits, I + H, xh)
    h_ref, c_ref = po.lstm_pointwise(Y, bias, c)
    for lay in (GATES, LAYOUTS["mfma"]):
        lin = pb.PackedLinear(dev(W), bits, max_batch=N, layout=lay)
        h_out = torch.empty((N, H), dtype=torch.float32, device="cuda")
        c_out = torch.empty((N, H), dtype=torch.float32, device="cuda")
        pb.pb_lstm_cell(lin.packed, lin.scales, lin.desc, bits, dev(x), I, dev(h), dev(c), dev(bias), h_out, c_out, N,
                        lin.workspace)
        assert np.abs(h_out.cpu().numpy() - h_ref).max() <= 2e-6
        assert np.abs(c_out.cpu().numpy() - c_ref).max() <= 2e-6


GATES = 0x50420003


@pytest.mark.parametrize("mode,bits", [(1, 1), (1, 3), (1, 8), (2, 2), (3, 1), (3, 2), (3, 4), (3, 8)])
def test_quantizer_variants_match_the_oracle(pb, layout, mode, bits):
    """Section 3.3's other quantizers: codes and scales bit-exact, then the product on top of them."""
    rng = np.random.default_rng(100 * mode + bits)
    for (R, C) in [(37, 200), (300, 1000)]:
        W = rng.normal(0, 0.05, size=(R, C)).astype(np.float32)
        W[3, 5] = 0.9                                  # an outlier, so that the clipping search clips
        if mode == 1:
            W += np.float32(0.02)                      # not symmetric: max - min differs from 2 max|W|
        X = rng.normal(size=(2, C)).astype(np.float32)
        prep = po.prepare(W, bits, mode)
        lin = pb.PackedLinear(dev(W), bits, max_batch=2, layout=layout, quantizer=mode)
        assert (lin.unpack().cpu().numpy() == prep["q"]).all(), (mode, bits, R, C)
        assert (lin.scales[:bits].cpu().numpy().view(np.int32) == prep["scales"].view(np.int32)).all()
        lw = po.pack_words(prep["layers"])
        A_ref, Y_ref = po.matmul_words(lw, prep["scales"], bits, C, X)
        assert (lin.acc(dev(X), bits).cpu().numpy() == A_ref).all()
        assert_y_close(lin(dev(X), bits).cpu().numpy(), Y_ref, A_ref, prep["scales"])


def test_quantizer_mode_arguments(pb):
    d = pb.pb_desc_init(8, 64, 3)
    W = torch.zeros((8, 64), device="cuda")
    packed = pb.alloc_packed(d)
    sc = torch.zeros(4, device="cuda")
    with pytest.raises(pb.PbError) as e:
        pb.pb_quantize_pack_mode(W, d, 2, packed, sc)          # the +-1 code needs bits = 2
    assert e.value.status == pb.PB_EINVAL
    with pytest.raises(pb.PbError) as e:
        pb.pb_quantize_pack_mode(W, d, 7, packed, sc)
    assert e.value.status == pb.PB_EINVAL
    # all-zero weights: step 1 (0 for the +-1 code), codes 0
    for mode in (0, 1, 3):
        pb.pb_quantize_pack_mode(W, d, mode, packed, sc)
        assert sc[:3].cpu().tolist() == [-4.0, 2.0, 1.0]


@pytest.mark.parametrize("H,I,batch", [(5, 3, 1), (37, 100, 2), (64, 64, 4), (1500, 1500, 1)])
def test_gate_interleaved_layout_is_transparent(pb, H, I, batch):
    """The LSTM layout stores rows gate-interleaved; codes, accumulators and outputs come back in matrix order."""
    W, X = synth.ragged(4 * H, I + H, batch=batch, case=13, xdist="uniform")
    print("gates layout", H, I, batch, flush=True)
    run_layer(pb, W, 4, X, [1, 3, 4], layout=GATES)


def test_gate_layout_needs_rows_multiple_of_4(pb):
    with pytest.raises(pb.PbError) as e:
        pb.pb_desc_init_layout(10, 64, 4, GATES)
    assert e.value.status in (pb.PB_EINVAL, pb.PB_ESIZE)


@pytest.mark.parametrize("lay", ["mfma", "popc", "pair"])
@pytest.mark.parametrize("act", [0, 1])
def test_bias_and_relu_epilogue(pb, lay, act):
    W, X = synth.ragged(123, 900, batch=3, case=17, xdist="normal")
    bits, m = 5, 4
    rng = np.random.default_rng(17)
    bias = rng.normal(size=123).astype(np.float32)
    lin = pb.PackedLinear(dev(W), bits, max_batch=3, layout=LAYOUTS[lay])
    ref = oracle_reference(W, bits, X, m)
    want = ref["Y"] + bias[None, :]                      # fp32 add, as in the kernel
    if act:
        want = np.maximum(want, np.float32(0))
    Y = torch.empty((3, 123), dtype=torch.float32, device="cuda")
    pb.pb_matmul_bias_act(lin.packed, lin.scales, lin.desc, m, dev(X), 3, dev(bias), act, Y, lin.workspace)
    got = Y.cpu().numpy()
    tol = 1e-5 * np.abs(ref["Y"]) + 1e-6 * np.abs(bias[None, :]) + 1e-30
    assert (np.abs(got - want) <= tol).all()
    # without bias
    pb.pb_matmul_bias_act(lin.packed, lin.scales, lin.desc, m, dev(X), 3, None, act, Y, lin.workspace)
    want = np.maximum(ref["Y"], np.float32(0)) if act else ref["Y"]
    assert_y_close(Y.cpu().numpy(), want, ref["A"], ref["scales"])


def test_lstm_fused_cell_small_ragged(pb):
    """Fused product + cell update (one launch) on shapes whose H is not a multiple of 4 and with a batch."""
    for (H, I, N) in [(5, 7, 1), (38, 50, 3), (130, 70, 2), (37, 33, 1), (21, 1001, 2), (300, 2, 1), (38, 50, 6),
                      (21, 1001, 11), (9, 515, 8)]:
        W, X = synth.ragged(4 * H, I + H, batch=N, case=19, xdist="uniform")
        rng = np.random.default_rng(19)
        bias = rng.normal(size=4 * H).astype(np.float32) * 0.1
        c0 = rng.normal(size=(N, H)).astype(np.float32)
        x_t, h0 = X[:, :I].copy(), X[:, I:].copy()
        bits, m = 5, 5
        prep = po.prepare(W, bits)
        lw = po.pack_words(prep["layers"])
        _, Y_or = po.matmul_words(lw, prep["scales"], m, I + H, X)
        h_ref, c_ref = po.lstm_pointwise(Y_or, bias, c0)
        lin = pb.PackedLinear(dev(W), bits, max_batch=N, layout=GATES)
        h_out = torch.empty((N, H), device="cuda")
        c_out = torch.empty((N, H), device="cuda")
        pb.pb_lstm_cell(lin.packed, lin.scales, lin.desc, m, dev(x_t), I, dev(h0), dev(c0), dev(bias), h_out, c_out,
                        N, lin.workspace)
        assert np.abs(h_out.cpu().numpy() - h_ref).max() < 2e-6, (H, I, N)
        assert np.abs(c_out.cpu().numpy() - c_ref).max() < 2e-6, (H, I, N)


@pytest.mark.parametrize("layout", [LAYOUTS["mfma"], LAYOUTS["popc"], GATES, LAYOUTS["pair"]],
                         ids=["mfma", "popc", "gates", "pair"])
def test_lstm_cell_config4(pb, layout):
    """Config 4: 35 sequential LSTM steps.  Integer parity is checked per step with oracle-fed state
    (teacher forcing); the free-running GPU recurrence is compared to a tolerance."""
    H = I = 1500
    W, xs, bias = synth.lstm(H, I, steps=35)
    bits, m = 4, 4
    prep = po.prepare(W, bits)
    lw = po.pack_words(prep["layers"])
    lin = pb.PackedLinear(dev(W), bits, layout=layout)
    d, packed, scales, ws = lin.desc, lin.packed, lin.scales, lin.workspace
    bias_d = dev(bias)
    h_or = np.zeros((1, H), dtype=np.float32)
    c_or = np.zeros((1, H), dtype=np.float32)
    h_free = torch.zeros((1, H), device="cuda")
    c_free = torch.zeros((1, H), device="cuda")
    h_pp = [torch.zeros((1, H), device="cuda"), torch.zeros((1, H), device="cuda")]   # ping-pong (never aliased)
    c_pp = torch.zeros((1, H), device="cuda")
    for t in range(35):
        xin = np.concatenate([xs[t], h_or], axis=1)
        A_or, Y_or = po.matmul_words(lw, prep["scales"], m, I + H, xin)
        if t in (0, 1, 17, 34):
            A_gpu = lin.acc(dev(xin), m).cpu().numpy()
            assert (A_gpu == A_or).all(), "step %d" % t
        # one GPU step from the oracle's state
        h_in, c_in = dev(h_or), dev(c_or)
        h_out = torch.empty_like(h_in)
        c_out = torch.empty_like(c_in)
        pb.pb_lstm_cell(packed, scales, d, m, dev(xs[t]), I, h_in, c_in, bias_d, h_out, c_out, 1, ws)
        h_new, c_new = po.lstm_pointwise(Y_or, bias, c_or)
        assert np.abs(h_out.cpu().numpy() - h_new).max() < 2e-6, "step %d" % t
        assert np.abs(c_out.cpu().numpy() - c_new).max() < 2e-6, "step %d" % t
        # free-running GPU recurrence (in place)
        pb.pb_lstm_cell(packed, scales, d, m, dev(xs[t]), I, h_free, c_free, bias_d, h_free, c_free, 1, ws)
        pb.pb_lstm_cell(packed, scales, d, m, dev(xs[t]), I, h_pp[t & 1], c_pp, bias_d, h_pp[(t + 1) & 1], c_pp, 1, ws)
        h_or, c_or = h_new, c_new
    assert np.abs(h_free.cpu().numpy() - h_or).max() < 1e-4
    assert np.abs(c_free.cpu().numpy() - c_or).max() < 1e-4
    assert np.abs(h_pp[35 & 1].cpu().numpy() - h_or).max() < 1e-4
    assert np.abs(c_pp.cpu().numpy() - c_or).max() < 1e-4


def test_errors_surface_as_status(pb):
    d = pb.pb_desc_init(8, 64, 4)
    X = torch.zeros((1, 64), device="cuda")
    Y = torch.zeros((1, 8), device="cuda")
    packed = pb.alloc_packed(d)
    ws = pb.alloc_workspace(d, 1)
    sc = torch.zeros(4, device="cuda")
    with pytest.raises(pb.PbError) as e:
        pb.pb_matmul(packed, sc, d, 5, X, 1, Y, ws)
    assert e.value.status == pb.PB_EINVAL
    with pytest.raises(pb.PbError) as e:
        pb.pb_matmul(packed, sc, d, 4, X[:, 1:].contiguous()[:, :0].reshape(-1).new_zeros(65)[1:], 1, Y, ws)
    assert e.value.status == pb.PB_EALIGN


def test_calibration_loop_runs_and_rejects_bad_arguments(pb):
    from paper_2003_00822_amd import calib
    out = torch.zeros(4, dtype=torch.float32, device="cuda")
    for mode in (0, 1, 2):
        calib.pb_calib_mfma(mode, 3, 4, out)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    for bad in ((3, 1, 1), (0, 0, 1), (0, 1, 0)):
        with pytest.raises(Exception):
            calib.pb_calib_mfma(bad[0], bad[1], bad[2], out)


def test_graph_replay_matches_eager(pb):
    """A captured sequence of calls (two FC layers with bias + ReLU, then an LSTM step) replayed several times with
    new inputs and eager work in between gives the eager results bit for bit."""
    rng = np.random.default_rng(77)
    W1, X = synth.ragged(96, 300, batch=3, case=51, xdist="normal")
    W2, _ = synth.ragged(64, 96, batch=3, case=52)
    H = 16
    Wl, _ = synth.ragged(4 * H, 64 + H, batch=3, case=53)
    l1 = pb.PackedLinear(dev(W1), 6, max_batch=3)
    l2 = pb.PackedLinear(dev(W2), 4, max_batch=3)
    ll = pb.PackedLinear(dev(Wl), 5, max_batch=3, layout=GATES)
    b1 = dev(rng.normal(size=96).astype(np.float32))
    b2 = dev(rng.normal(size=64).astype(np.float32))
    bl = dev(rng.normal(size=4 * H).astype(np.float32))
    x = dev(X)
    y1 = torch.empty((3, 96), device="cuda")
    y2 = torch.empty((3, 64), device="cuda")
    h = torch.zeros((3, H), device="cuda")
    c = torch.zeros((3, H), device="cuda")
    h_out = torch.empty_like(h)
    c_out = torch.empty_like(c)

    def forward():
        pb.pb_matmul_bias_act(l1.packed, l1.scales, l1.desc, 5, x, 3, b1, pb.PB_ACT_RELU, y1, l1.workspace)
        pb.pb_matmul_bias_act(l2.packed, l2.scales, l2.desc, 4, y1, 3, b2, pb.PB_ACT_NONE, y2, l2.workspace)
        pb.pb_lstm_cell(ll.packed, ll.scales, ll.desc, 5, y2, 64, h, c, bl, h_out, c_out, 3, ll.workspace)

    forward()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        forward()
    for it in range(4):
        x.copy_(dev(rng.normal(size=X.shape).astype(np.float32)))
        h.copy_(dev(rng.normal(size=(3, H)).astype(np.float32)))
        c.copy_(dev(rng.normal(size=(3, H)).astype(np.float32)))
        g.replay()
        torch.cuda.synchronize()
        got = (y2.clone(), h_out.clone(), c_out.clone())
        junk = torch.randn(1 << 16, device="cuda").sum()   # eager work between the replays
        forward()
        torch.cuda.synchronize()
        assert torch.isfinite(junk)
        for a_, b_ in zip(got, (y2, h_out, c_out)):
            assert torch.equal(a_, b_), "replay %d differs from the eager run" % it


def test_graph_replay_of_wide_rows(pb):
    """The kernels that take wide rows in several passes keep sums in LDS from pass to pass: a captured call (9000
    columns, batch 6, 70 row tiles) replayed with new inputs, eager calls of other shapes in between, gives the eager
    result bit for bit."""
    rng = np.random.default_rng(78)
    W, X = synth.ragged(1100, 9000, batch=6, case=54, xdist="normal")
    lin = pb.PackedLinear(dev(W), 6, max_batch=6, layout=LAYOUTS["pair"])
    Ws, Xs = synth.ragged(40, 700, batch=2, case=55)
    small = pb.PackedLinear(dev(Ws), 4, max_batch=2)
    x = dev(X)
    xs = dev(Xs)
    y = torch.empty((6, 1100), device="cuda")
    bias = dev(rng.normal(size=1100).astype(np.float32))

    def call():
        pb.pb_matmul_bias_act(lin.packed, lin.scales, lin.desc, 5, x, 6, bias, pb.PB_ACT_RELU, y, lin.workspace)

    call()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for it in range(4):
        x.copy_(dev(rng.normal(size=X.shape).astype(np.float32)))
        g.replay()
        torch.cuda.synchronize()
        got = y.clone()
        small(xs, 3)                                        # other work between the replays
        call()
        torch.cuda.synchronize()
        assert torch.equal(got, y), "replay %d differs from the eager run" % it
    ref = oracle_reference(W, 6, x.cpu().numpy(), 5)
    want = np.maximum(ref["Y"] + bias.cpu().numpy()[None, :], 0)
    assert np.abs(y.cpu().numpy() - want).max() <= 1e-5 * np.abs(want).max()

