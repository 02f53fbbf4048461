"""Host logic of the packed layouts (csrc/pb_layout.h), compiled for the CPU: sizes, padding, and that the
position of every (bitlayer, row, word) is unique and follows the block structure the kernels rely on."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ROWMAJOR, TILE16, GATES = 0x50420001, 0x50420002, 0x50420003


@pytest.fixture(scope="module")
def probe(tmp_path_factory):
    out = tmp_path_factory.mktemp("layout") / "liblayout_probe.so"
    cmd = ["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-D__host__=", "-D__device__=",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2003_00822_amd", "csrc"),
           "-o", str(out), os.path.join(ROOT, "tests", "layout_probe.cpp")]
    subprocess.check_call(cmd)
    L = ctypes.CDLL(str(out))
    L.probe_layout.restype = ctypes.c_longlong
    L.probe_layout.argtypes = [ctypes.c_uint, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
    L.probe_word_index.restype = ctypes.c_longlong
    L.probe_word_index.argtypes = [ctypes.c_uint, ctypes.c_int, ctypes.c_longlong, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_int]
    L.probe_packed_bytes.restype = ctypes.c_longlong
    L.probe_workspace_bytes.restype = ctypes.c_longlong
    return L


def layout_of(probe, layout, rows, cols, bits):
    out = (ctypes.c_int * 10)()
    lw = probe.probe_layout(layout, rows, cols, bits, out)
    names = ["cw", "cwp", "rows_p", "rt_count", "cq", "gate_h", "ws", "csplit", "rpt", "ok"]
    d = dict(zip(names, list(out)))
    d["layer_words"] = lw
    return d


def test_tiled_layout_sizes_and_padding(probe):
    L = layout_of(probe, TILE16, 100, 3000, 3)
    assert (L["cw"], L["cwp"], L["rows_p"], L["rt_count"], L["cq"]) == (94, 96, 112, 7, 6)
    assert L["layer_words"] == 112 * 96
    assert probe.probe_packed_bytes(TILE16, 100, 3000, 3) == 3 * 112 * 96 * 4
    L = layout_of(probe, TILE16, 1, 1, 1)
    assert (L["cwp"], L["rows_p"]) == (16, 16)
    L = layout_of(probe, TILE16, 16, 32768, 16)
    assert L["ok"] == 1 and L["cq"] == 64
    assert layout_of(probe, TILE16, 16, 32769, 1)["ok"] == 0
    assert layout_of(probe, TILE16, 16, 64, 17)["ok"] == 0
    assert layout_of(probe, TILE16, 0, 64, 1)["ok"] == 0


PAIRS = 0x50420004


def test_pairs_layout_sizes(probe):
    """The layout with the digits of the bitlayer pairs has the blocks of the tiled layout and room for an even
    number of bitlayers (a last single one is paired with zeros)."""
    for bits, stored in ((1, 2), (2, 2), (3, 4), (8, 8), (15, 16), (16, 16)):
        assert probe.probe_packed_bytes(PAIRS, 100, 3000, bits) == stored * 112 * 96 * 4
        assert layout_of(probe, PAIRS, 100, 3000, bits) == layout_of(probe, TILE16, 100, 3000, bits)
    assert probe.probe_workspace_bytes(PAIRS, 100, 3000, 3, 5) == probe.probe_workspace_bytes(TILE16, 100, 3000, 3, 5)


def test_pair_digit_words(probe):
    """Digit d_c = 2 upper_c + lower_c of column c: two bits at c, c + 1 of the even word (c even), at c - 1, c of
    the odd word (c odd).  Worked by hand for a few patterns, then against the definition, and back."""
    out = (ctypes.c_uint * 4)()
    probe.probe_pair_digits(0b0110, 0b0011, out)       # columns 0..3: digits 1, 3, 2, 0
    assert out[0] == (1 << 0) | (2 << 2)               # even columns 0, 2: digits 1 (bits 0-1), 2 (bits 2-3)
    assert out[1] == (3 << 0) | (0 << 2)               # odd columns 1, 3: digits 3 (bits 0-1), 0 (bits 2-3)
    assert (out[2], out[3]) == (0b0110, 0b0011)
    import random
    rng = random.Random(5)
    for _ in range(200):
        up, lo = rng.getrandbits(32), rng.getrandbits(32)
        probe.probe_pair_digits(up, lo, out)
        for c in range(32):
            d = 2 * ((up >> c) & 1) + ((lo >> c) & 1)
            word, pos = (out[0], c) if c % 2 == 0 else (out[1], c - 1)
            assert (word >> pos) & 3 == d
        assert (out[2], out[3]) == (up, lo)


def test_gate_layout_sizes(probe):
    L = layout_of(probe, GATES, 4 * 38, 88, 5)
    assert L["gate_h"] == 38 and L["rt_count"] == 10 and L["rows_p"] == 160      # four units per tile
    assert layout_of(probe, GATES, 10, 64, 4)["ok"] == 0                          # rows not a multiple of 4


def test_rowmajor_layout_sizes(probe):
    L = layout_of(probe, ROWMAJOR, 100, 3000, 3)
    assert L["cw"] == 94 and L["cwp"] == L["ws"] * L["csplit"] and L["cwp"] >= 94
    assert L["rows_p"] == 100 and L["rpt"] * L["ws"] == 128
    L = layout_of(probe, ROWMAJOR, 10, 784, 2)
    assert (L["cwp"], L["rows_p"]) == (32, 12)


@pytest.mark.parametrize("layout", [ROWMAJOR, TILE16])
@pytest.mark.parametrize("shape", [(1, 1, 1), (5, 33, 2), (37, 1000, 3), (16, 512, 1), (50, 2100, 4)])
def test_word_positions_are_a_bijection(probe, layout, shape):
    rows, cols, bits = shape
    L = layout_of(probe, layout, rows, cols, bits)
    seen = np.zeros(L["layer_words"] * bits, dtype=np.uint8)
    for layer in range(bits):
        for r in range(L["rows_p"]):
            for w in range(L["cwp"]):
                i = probe.probe_word_index(layout, L["cwp"], L["layer_words"], layer, r, w)
                assert 0 <= i < seen.size
                assert layer * L["layer_words"] <= i < (layer + 1) * L["layer_words"]    # bitlayers are contiguous
                seen[i] += 1
    assert (seen == 1).all()


def test_tiled_block_structure(probe):
    """A 1 KB block = 16 rows x 16 words of one (row tile, chunk): lane 16 kb + j owns the 16 bytes at 16 lane, words
    4 kb + t of row j; blocks of one row tile follow each other chunk by chunk, row tiles follow each other."""
    rows, cols, bits = 40, 1500, 2
    L = layout_of(probe, TILE16, rows, cols, bits)
    cq = L["cq"]
    for layer in range(bits):
        for r in range(L["rows_p"]):
            for w in range(L["cwp"]):
                i = probe.probe_word_index(TILE16, L["cwp"], L["layer_words"], layer, r, w)
                rt, j, q, kb, t = r // 16, r % 16, w // 16, (w % 16) // 4, w % 4
                block = rt * cq + q
                want = layer * L["layer_words"] + block * 256 + (16 * kb + j) * 4 + t
                assert i == want


def test_gate_row_mapping_is_a_bijection(probe):
    for H in (1, 3, 4, 5, 38, 1500):
        tiles = (H + 3) // 4
        seen = set()
        for gate in range(4):
            for u in range(H):
                pr = probe.probe_gates_packed_row(gate * H + u, H)
                assert pr == (u // 4) * 16 + (u % 4) * 4 + gate          # the four gates of a unit are adjacent
                assert 0 <= pr < 16 * tiles and pr not in seen
                seen.add(pr)
                assert probe.probe_gates_matrix_row(pr, H) == gate * H + u
        for pr in range(16 * tiles):
            if pr not in seen:
                assert probe.probe_gates_matrix_row(pr, H) == -1             # padding rows


def test_workspace_grows_with_batch(probe):
    a = probe.probe_workspace_bytes(TILE16, 100, 3000, 3, 1)
    b = probe.probe_workspace_bytes(TILE16, 100, 3000, 3, 7)
    assert a > 0 and b > a and a % 256 == 0 and b % 256 == 0



def test_passes_over_wide_rows(probe):
    """The geometry that the launcher and the matrix-core kernel share when batches on wide rows take the columns
    in several passes (of what eight waves hold: 16 chunks with two chunks per wave, 8 with one): every chunk belongs
    to exactly one pass, a pass never has more chunks than its capacity, the passes are as few as that allows and
    evenly filled, and a row within the capacity needs one."""
    caps = (ctypes.c_int * 2)()
    probe.probe_split_caps(caps)
    assert list(caps) == [16, 8]
    out = (ctypes.c_int * 2)()
    widest = layout_of(probe, TILE16, 16, 32768, 8)["cq"]
    assert widest == 64
    for cap, per_wave in ((16, 2), (8, 1)):
        for cq in range(1, widest + 1):
            probe.probe_split(cq, cap, out)
            parts, per = list(out)
            assert parts == -(-cq // cap) and 1 <= parts <= widest // cap
            assert per <= cap and parts * per >= cq > (parts - 1) * per
            waves = -(-per // per_wave)
            assert 1 <= waves <= 8
            # wave w of pass p owns per_wave chunks from per_wave (p * waves + w): all chunks once, in order
            owned = [per_wave * (p * waves + w) + k for p in range(parts) for w in range(waves) for k in range(per_wave)]
            assert sorted(set(owned)) == owned and set(range(cq)) <= set(owned)
