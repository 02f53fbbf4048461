"""Loader of the benchmark's calibration loop (`csrc/calib/pb_calib.hip`, `libpbatch_calib.so`): a loop of the
product kernel's FP4 matrix instruction on constant operands, which `bench.py` times to state what fraction of the
matrix peak is reachable beside the kernel's vector-ALU work.  Not a step of the method and not part of the C ABI
of the product library."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        path = os.environ.get("PBATCH_CALIB_LIB", os.path.join(_HERE, "libpbatch_calib.so"))
        if not os.path.exists(path):
            raise RuntimeError("%s is missing: run `python -m paper_2003_00822_amd.build`" % path)
        L = ctypes.CDLL(path)
        L.pb_calib_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        L.pb_calib_mfma.restype = ctypes.c_int
        _LIB = L
    return _LIB


def pb_calib_mfma(mode, iters, workgroups, out, stream=None):
    """mode 0: the instructions alone; 1: with the expansion of a packed weight word per four instructions; 2: also
    with an epilogue per chain of four.  `out`: fp32 CUDA tensor of `workgroups` elements (a checksum)."""
    import torch
    if not (isinstance(out, torch.Tensor) and out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
            and out.numel() >= max(workgroups, 1)):
        raise ValueError("out: contiguous fp32 CUDA tensor of at least `workgroups` elements")
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    rc = lib().pb_calib_mfma(mode, iters, workgroups, ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(st))
    if rc != 0:
        raise RuntimeError("pb_calib_mfma: %s" % ("arguments out of range" if rc == 1 else "launch failed"))
