"""The entry point that allocates nothing (pb_matmul_static: the workspace lives in a device array of the library)
against pb_matmul, through the C ABI: same kernels, so the outputs must be identical bit for bit; two calls in a
row, the second with a smaller input, on the layout whose kernels use the workspace and on the two tiled ones."""
import ctypes

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import pb_oracle as po
from paper_2003_00822_amd import synth
from tests.helpers import assert_y_close, oracle_reference

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pb():
    assert torch.cuda.is_available(), "gpu tests need a GPU"
    from paper_2003_00822_amd import pb as _pb
    _pb.lib()  # fails loudly if the HIP library is missing
    return _pb


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def raw_static(pb, lin, X, m, Y):
    """pb_matmul_static through ctypes on raw device pointers (no workspace argument)."""
    L = pb.lib()
    rc = L.pb_matmul_static(ctypes.c_void_p(lin.packed.data_ptr()), ctypes.c_void_p(lin.scales.data_ptr()),
                            ctypes.byref(lin.desc), m, ctypes.c_void_p(X.data_ptr()), X.shape[0],
                            ctypes.c_void_p(Y.data_ptr()), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    return rc


@pytest.mark.parametrize("layout_name", ["popc", "mfma", "pair"])
def test_static_scratch_matches_pb_matmul_twice(pb, layout_name):
    layout = {"popc": pb.PB_LAYOUT_ROWMAJOR_V1, "mfma": pb.PB_LAYOUT_TILE16_V1,
              "pair": pb.PB_LAYOUT_TILE16_PAIRS_V1}[layout_name]
    bits = 6
    # first call: 300 x 2100, batch 5; then rows wide enough for the kernels that take the columns in two passes;
    # last a smaller matrix and batch (the scratch keeps the earlier calls' planes)
    for (R, C, N, m, case) in ((300, 2100, 5, 6, 61), (90, 9000, 6, 5, 63), (70, 500, 2, 3, 62)):
        print("static scratch", layout_name, R, C, N, flush=True)
        W, X = synth.ragged(R, C, batch=N, case=case, xdist="wide")
        lin = pb.PackedLinear(dev(W), bits, max_batch=N, layout=layout)
        Xd = dev(X)
        Y_ws = torch.empty((N, R), dtype=torch.float32, device="cuda")
        pb.pb_matmul(lin.packed, lin.scales, lin.desc, m, Xd, N, Y_ws, lin.workspace)
        Y_st = torch.full((N, R), float("nan"), dtype=torch.float32, device="cuda")
        assert raw_static(pb, lin, Xd, m, Y_st) == pb.PB_OK
        torch.cuda.synchronize()
        a, b = Y_ws.cpu().numpy(), Y_st.cpu().numpy()
        assert (a.view(np.int32) == b.view(np.int32)).all()
        ref = oracle_reference(W, bits, X, m)
        assert_y_close(b, ref["Y"], ref["A"], ref["scales"])
        # the binding of the same name
        Y_b = torch.empty_like(Y_st)
        pb.pb_matmul_static(lin.packed, lin.scales, lin.desc, m, Xd, N, Y_b)
        assert (Y_b.cpu().numpy().view(np.int32) == a.view(np.int32)).all()


def test_static_scratch_rejects_what_does_not_fit(pb):
    d = pb.pb_desc_init_layout(64, 32768, 4, pb.PB_LAYOUT_ROWMAJOR_V1)
    need = pb.lib().pb_workspace_bytes(ctypes.byref(d), 64)
    assert need > (2 << 20)
    fake = ctypes.c_void_p(0x1000)
    L = pb.lib()
    assert L.pb_matmul_static(fake, fake, ctypes.byref(d), 4, fake, 64, fake, None) == pb.PB_ESIZE
    assert L.pb_matmul_static(fake, fake, ctypes.byref(d), 4, fake, 0, fake, None) == pb.PB_EINVAL
    assert L.pb_matmul_static(fake, fake, ctypes.byref(d), 4, fake, 1, None, None) == pb.PB_EINVAL
    assert L.pb_matmul_static(fake, fake, ctypes.byref(d), 5, fake, 1, fake, None) == pb.PB_EINVAL     # bits_used > bits
    assert L.pb_matmul_static(None, fake, ctypes.byref(d), 4, fake, 1, fake, None) == pb.PB_EINVAL
