"""Host-side checks of the C-ABI library: it loads, exports every symbol the header declares,
answers size queries and rejects bad arguments before launching anything (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pb():
    from paper_2003_00822_amd import pb as pbmod
    if not os.path.exists(pbmod.LIB_PATH):
        from paper_2003_00822_amd import build
        build.build(verbose=False)
    return pbmod


def declared_functions():
    names = []
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(pb_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_header_symbols_exported(pb):
    L = pb.lib()
    names = declared_functions()
    assert "pb_quantize_pack" in names and "pb_matmul" in names and "pb_lstm_cell" in names
    for n in names:
        assert hasattr(L, n), "library does not export %s" % n
    assert sorted(pb.EXPORTS) == names


def test_desc_and_sizes(pb):
    d = pb.pb_desc_init(4096, 4096, 8)
    assert (d.rows, d.cols, d.bits, d.frac_bits, d.act_bits) == (4096, 4096, 8, 16, 32)
    assert d.layout == pb.PB_LAYOUT_TILE16_V1
    assert pb.pb_packed_bytes(d) == 8 * 4096 * 4096 // 8
    # tiled layout, ragged: rows padded to 16, words per row to 16
    d = pb.pb_desc_init(100, 3000, 3)
    assert pb.pb_packed_bytes(d) == 3 * 112 * 96 * 4
    d = pb.pb_desc_init(10, 784, 2)
    assert pb.pb_packed_bytes(d) == 2 * 16 * 32 * 4
    # row-major layout, ragged: 100 x 3000 -> rows padded to 100, words per row padded to 96
    d = pb.pb_desc_init_layout(100, 3000, 3, pb.PB_LAYOUT_ROWMAJOR_V1)
    assert pb.pb_packed_bytes(d) == 3 * 100 * 96 * 4
    d = pb.pb_desc_init_layout(10, 784, 2, pb.PB_LAYOUT_ROWMAJOR_V1)
    assert pb.pb_packed_bytes(d) == 2 * 12 * 32 * 4
    # the tiled layout is the default at every width
    assert pb.pb_desc_init(8, pb.PB_MAX_COLS, 2).layout == pb.PB_LAYOUT_TILE16_V1
    assert pb.pb_packed_bytes(pb.pb_desc_init(8, 16385, 2)) == 2 * 16 * 528 * 4
    with pytest.raises(pb.PbError) as e:
        pb.pb_desc_init_layout(8, 64, 2, 7)
    assert e.value.status == pb.PB_EINVAL
    ws1 = pb.pb_workspace_bytes(d, 1)
    ws4 = pb.pb_workspace_bytes(d, 4)
    assert ws1 >= 32 * 32 * 4 + 10 * 4 and ws4 > ws1
    assert pb.pb_workspace_bytes(d, 0) == 0
    assert pb.pb_workspace_bytes(d, pb.PB_MAX_BATCH + 1) == 0


@pytest.mark.parametrize("args", [(0, 8, 4), (8, 0, 4), (8, 8, 0), (8, 8, 17), (-1, 8, 4)])
def test_desc_init_rejects(pb, args):
    with pytest.raises(pb.PbError) as e:
        pb.pb_desc_init(*args)
    assert e.value.status == pb.PB_EINVAL


def test_desc_init_size_limit(pb):
    with pytest.raises(pb.PbError) as e:
        pb.pb_desc_init(8, pb.PB_MAX_COLS + 1, 4)
    assert e.value.status == pb.PB_ESIZE
    pb.pb_desc_init(8, pb.PB_MAX_COLS, 4)


def test_null_and_range_arguments_rejected_before_launch(pb):
    L = pb.lib()
    d = pb.pb_desc_init(64, 64, 4)
    dp = ctypes.byref(d)
    fake = ctypes.c_void_p(0x1000)       # aligned, never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1004)
    null = ctypes.c_void_p(0)
    assert L.pb_quantize_pack(null, 64, 64, 4, fake, fake, null) == pb.PB_EINVAL
    assert L.pb_quantize_pack(fake, 64, 64, 0, fake, fake, null) == pb.PB_EINVAL
    assert L.pb_quantize_pack(odd, 64, 64, 4, fake, fake, null) == pb.PB_EALIGN
    assert L.pb_matmul(fake, fake, dp, 0, fake, 1, fake, fake, null) == pb.PB_EINVAL      # bits_used < 1
    assert L.pb_matmul(fake, fake, dp, 5, fake, 1, fake, fake, null) == pb.PB_EINVAL      # bits_used > bits
    assert L.pb_matmul(fake, fake, dp, 4, fake, 0, fake, fake, null) == pb.PB_EINVAL      # batch < 1
    assert L.pb_matmul(fake, fake, dp, 4, fake, pb.PB_MAX_BATCH + 1, fake, fake, null) == pb.PB_ESIZE
    assert L.pb_matmul(fake, fake, dp, 4, null, 1, fake, fake, null) == pb.PB_EINVAL      # X null
    assert L.pb_matmul(fake, fake, dp, 4, fake, 1, null, fake, null) == pb.PB_EINVAL      # Y null
    assert L.pb_matmul(fake, fake, dp, 4, fake, 1, fake, null, null) == pb.PB_EINVAL      # workspace null
    assert L.pb_matmul(fake, fake, dp, 4, odd, 1, fake, fake, null) == pb.PB_EALIGN
    assert L.pb_matmul(fake, fake, None, 4, fake, 1, fake, fake, null) == pb.PB_EINVAL    # desc null
    assert L.pb_matmul_acc(fake, dp, 4, fake, 1, null, fake, null) == pb.PB_EINVAL
    assert L.pb_unpack(null, dp, fake, null) == pb.PB_EINVAL
    assert L.pb_fixed_point(dp, fake, 1, null, fake, null) == pb.PB_EINVAL
    bad = pb.pb_desc_init(64, 64, 4)
    bad.layout = 7
    assert L.pb_matmul(fake, fake, ctypes.byref(bad), 4, fake, 1, fake, fake, null) == pb.PB_EINVAL
    bad = pb.pb_desc_init(64, 64, 4)
    bad.act_bits = 33
    assert L.pb_matmul(fake, fake, ctypes.byref(bad), 4, fake, 1, fake, fake, null) == pb.PB_EINVAL
    # LSTM shape rules: rows = 4H, cols = I + H
    dl = pb.pb_desc_init(64, 48, 4)      # H = 16, so I must be 32
    dlp = ctypes.byref(dl)
    assert L.pb_lstm_cell(fake, fake, dlp, 4, fake, 31, fake, fake, null, fake, fake, 1, fake, null) == pb.PB_EINVAL
    d3 = pb.pb_desc_init(66, 48, 4)      # rows not a multiple of 4
    assert L.pb_lstm_cell(fake, fake, ctypes.byref(d3), 4, fake, 32, fake, fake, null, fake, fake, 1, fake,
                          null) == pb.PB_EINVAL


def test_gate_interleaved_layout_sizes_and_checks(pb):
    gates = pb.PB_LAYOUT_TILE16_GATES_V1
    # H = 1500: 375 row tiles of 4 hidden units (16 gate rows), 3000 columns -> 6 chunks of 16 words
    d = pb.pb_desc_init_layout(6000, 3000, 4, gates)
    assert pb.pb_packed_bytes(d) == 4 * 375 * 16 * 96 * 4
    # H = 5: two row tiles, the second one mostly padding
    d = pb.pb_desc_init_layout(20, 12, 2, gates)
    assert pb.pb_packed_bytes(d) == 2 * 2 * 16 * 16 * 4
    with pytest.raises(pb.PbError):
        pb.pb_desc_init_layout(10, 64, 4, gates)          # rows not a multiple of 4


def test_pairs_layout_sizes(pb):
    pairs = pb.PB_LAYOUT_TILE16_PAIRS_V1
    d = pb.pb_desc_init_layout(100, 3000, 8, pairs)
    assert d.layout == pairs and pb.pb_packed_bytes(d) == 8 * 112 * 96 * 4
    # an odd number of bitlayers is stored as the next even number (the last one paired with zeros)
    d = pb.pb_desc_init_layout(100, 3000, 5, pairs)
    assert d.bits == 5 and pb.pb_packed_bytes(d) == 6 * 112 * 96 * 4
    assert pb.pb_workspace_bytes(d, 3) == pb.pb_workspace_bytes(pb.pb_desc_init(100, 3000, 5), 3)
    with pytest.raises(pb.PbError):
        pb.pb_desc_init_layout(8, pb.PB_MAX_COLS + 1, 2, pairs)


def test_bias_act_arguments_rejected_before_launch(pb):
    L = pb.lib()
    d = pb.pb_desc_init(64, 64, 4)
    dp = ctypes.byref(d)
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    null = ctypes.c_void_p(0)
    assert L.pb_matmul_bias_act(fake, fake, dp, 4, fake, 1, null, 2, fake, fake, null) == pb.PB_EINVAL   # bad activation
    assert L.pb_matmul_bias_act(fake, fake, dp, 4, fake, 1, odd, 1, fake, fake, null) == pb.PB_EALIGN    # bias alignment
    assert L.pb_matmul_bias_act(fake, fake, dp, 4, fake, 1, null, 1, null, fake, null) == pb.PB_EINVAL   # Y null
    assert L.pb_matmul_bias_act(fake, fake, dp, 5, fake, 1, null, 0, fake, fake, null) == pb.PB_EINVAL   # bits_used


def test_pair_hook_arguments_rejected_before_launch(pb):
    L = pb.lib()
    fake = ctypes.c_void_p(0x1000)
    null = ctypes.c_void_p(0)
    d = pb.pb_desc_init_layout(64, 64, 4, pb.PB_LAYOUT_ROWMAJOR_V1)
    # the popcount layout has no bitlayer pairs
    assert L.pb_matmul_acc_pairs(fake, ctypes.byref(d), 4, fake, 1, fake, fake, null) == pb.PB_EINVAL
    d = pb.pb_desc_init(64, 64, 4)
    assert L.pb_matmul_acc_pairs(fake, ctypes.byref(d), 4, fake, 1, null, fake, null) == pb.PB_EINVAL    # A null
    assert L.pb_matmul_acc_pairs(fake, ctypes.byref(d), 0, fake, 1, fake, fake, null) == pb.PB_EINVAL    # bits_used
    assert L.pb_matmul_acc_pairs(fake, ctypes.byref(d), 4, fake, 0, fake, fake, null) == pb.PB_EINVAL    # batch


def test_calibration_loop_is_not_in_the_product_library_and_rejects_bad_arguments(pb):
    """The benchmark's calibration loop lives in a library of its own; arguments out of range launch nothing."""
    from paper_2003_00822_amd import calib
    assert not hasattr(pb.lib(), "pb_calib_mfma")
    C = calib.lib()
    fake = ctypes.c_void_p(0x1000)
    null = ctypes.c_void_p(0)
    for mode, iters, wgs, out in ((3, 1, 1, fake), (-1, 1, 1, fake), (0, 0, 1, fake), (0, 1, 0, fake),
                                  (0, 1, 1, null), (0, (1 << 20) + 1, 1, fake), (0, 1, 65537, fake)):
        assert C.pb_calib_mfma(mode, iters, wgs, out, null) == 1


def test_strerror(pb):
    assert pb.strerror(0) == "ok"
    for s in (pb.PB_EINVAL, pb.PB_EALIGN, pb.PB_ESIZE, pb.PB_EHIP):
        assert pb.strerror(s) and pb.strerror(s) != "unknown status"
    assert pb.strerror(-99) == "unknown status"
