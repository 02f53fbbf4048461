"""Thin Python binding of the C ABI in include/pb.h (same names, argument marshalling only).

Every step of the path runs in the HIP kernels of libpbatch.so; torch is used for
device memory and streams.  There is no CPU fallback: if the library is not built the
first call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# PBATCH_LIB points the binding at another build of the same library (e.g. one compiled with other tuning macros)
LIB_PATH = os.environ.get("PBATCH_LIB") or os.path.join(_HERE, "libpbatch.so")

PB_OK, PB_EINVAL, PB_EALIGN, PB_ESIZE, PB_EHIP = 0, -1, -2, -3, -4
PB_MAX_BITS = 16
PB_MAX_COLS = 32768
PB_MAX_BATCH = 4096
PB_LAYOUT_ROWMAJOR_V1 = 0x50420001   # AND + popcount kernel
PB_LAYOUT_TILE16_V1 = 0x50420002     # matrix-core kernel (what pb_desc_init picks)
PB_LAYOUT_TILE16_GATES_V1 = 0x50420003   # the same with the four gate rows of an LSTM unit in one row tile
PB_LAYOUT_TILE16_PAIRS_V1 = 0x50420004   # the same with two bitlayers per word as base-4 digits (for serving batches)
PB_ACT_NONE, PB_ACT_RELU = 0, 1
PB_QUANT_SYMMETRIC, PB_QUANT_RANGE, PB_QUANT_SIGN, PB_QUANT_CLIP_SEARCH = 0, 1, 2, 3

EXPORTS = [
    "pb_desc_init", "pb_desc_init_layout", "pb_quantize_pack_desc", "pb_quantize_pack_mode", "pb_packed_bytes", "pb_workspace_bytes", "pb_quantize_pack", "pb_unpack", "pb_matmul",
    "pb_matmul_static", "pb_matmul_bias_act", "pb_matmul_acc", "pb_matmul_acc_pairs", "pb_act_prep", "pb_matmul_prepared", "pb_fixed_point", "pb_lstm_cell", "pb_strerror", "pb_last_hip_error",
]


class pb_desc(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int32), ("cols", ctypes.c_int32), ("bits", ctypes.c_int32),
                ("frac_bits", ctypes.c_int32), ("act_bits", ctypes.c_int32), ("layout", ctypes.c_uint32)]


class PbError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, strerror(status), status))


_lib = None
_P = ctypes.c_void_p
_I = ctypes.c_int
_D = ctypes.POINTER(pb_desc)


def lib():
    """Load libpbatch.so (built by `python -m paper_2003_00822_amd.build`); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "HIP library %s is not built: run `python -m paper_2003_00822_amd.build` (no CPU fallback exists)"
                % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        L.pb_desc_init.argtypes = [_D, _I, _I, _I]
        L.pb_desc_init.restype = _I
        L.pb_desc_init_layout.argtypes = [_D, _I, _I, _I, ctypes.c_uint32]
        L.pb_desc_init_layout.restype = _I
        L.pb_quantize_pack_desc.argtypes = [_P, _D, _P, _P, _P]
        L.pb_quantize_pack_desc.restype = _I
        L.pb_quantize_pack_mode.argtypes = [_P, _D, _I, _P, _P, _P]
        L.pb_quantize_pack_mode.restype = _I
        L.pb_packed_bytes.argtypes = [_D]
        L.pb_packed_bytes.restype = ctypes.c_size_t
        L.pb_workspace_bytes.argtypes = [_D, _I]
        L.pb_workspace_bytes.restype = ctypes.c_size_t
        L.pb_quantize_pack.argtypes = [_P, _I, _I, _I, _P, _P, _P]
        L.pb_quantize_pack.restype = _I
        L.pb_unpack.argtypes = [_P, _D, _P, _P]
        L.pb_unpack.restype = _I
        L.pb_matmul.argtypes = [_P, _P, _D, _I, _P, _I, _P, _P, _P]
        L.pb_matmul.restype = _I
        L.pb_matmul_static.argtypes = [_P, _P, _D, _I, _P, _I, _P, _P]
        L.pb_matmul_static.restype = _I
        L.pb_matmul_bias_act.argtypes = [_P, _P, _D, _I, _P, _I, _P, _I, _P, _P, _P]
        L.pb_matmul_bias_act.restype = _I
        L.pb_matmul_acc.argtypes = [_P, _D, _I, _P, _I, _P, _P, _P]
        L.pb_matmul_acc.restype = _I
        L.pb_matmul_acc_pairs.argtypes = [_P, _D, _I, _P, _I, _P, _P, _P]
        L.pb_matmul_acc_pairs.restype = _I
        L.pb_act_prep.argtypes = [_D, _P, _I, _P, _P]
        L.pb_act_prep.restype = _I
        L.pb_matmul_prepared.argtypes = [_P, _P, _D, _I, _I, _P, _P, _P]
        L.pb_matmul_prepared.restype = _I
        L.pb_fixed_point.argtypes = [_D, _P, _I, _P, _P, _P]
        L.pb_fixed_point.restype = _I
        L.pb_lstm_cell.argtypes = [_P, _P, _D, _I, _P, _I, _P, _P, _P, _P, _P, _I, _P, _P]
        L.pb_lstm_cell.restype = _I
        L.pb_strerror.argtypes = [_I]
        L.pb_strerror.restype = ctypes.c_char_p
        L.pb_last_hip_error.argtypes = []
        L.pb_last_hip_error.restype = _I
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().pb_strerror(int(status)).decode()


def _check(status, where):
    if status != PB_OK:
        raise PbError(status, where)


def _ptr(t, dtype, name):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a CUDA/HIP tensor" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


def pb_desc_init(rows: int, cols: int, bits: int, frac_bits: int = 16, act_bits: int = 32) -> pb_desc:
    d = pb_desc()
    _check(lib().pb_desc_init(ctypes.byref(d), rows, cols, bits), "pb_desc_init")
    d.frac_bits = frac_bits
    d.act_bits = act_bits
    return d


def pb_desc_init_layout(rows: int, cols: int, bits: int, layout: int, frac_bits: int = 16,
                        act_bits: int = 32) -> pb_desc:
    d = pb_desc()
    _check(lib().pb_desc_init_layout(ctypes.byref(d), rows, cols, bits, layout), "pb_desc_init_layout")
    d.frac_bits = frac_bits
    d.act_bits = act_bits
    return d


def pb_packed_bytes(d: pb_desc) -> int:
    return int(lib().pb_packed_bytes(ctypes.byref(d)))


def pb_workspace_bytes(d: pb_desc, batch: int) -> int:
    return int(lib().pb_workspace_bytes(ctypes.byref(d), batch))


def alloc_packed(d: pb_desc, device="cuda") -> torch.Tensor:
    return torch.empty(pb_packed_bytes(d), dtype=torch.uint8, device=device)


def alloc_workspace(d: pb_desc, batch: int, device="cuda") -> torch.Tensor:
    return torch.empty(pb_workspace_bytes(d, batch), dtype=torch.uint8, device=device)


def pb_quantize_pack(W, rows, cols, bits, packed, scales, stream=None):
    _check(lib().pb_quantize_pack(_ptr(W, torch.float32, "W"), rows, cols, bits, _ptr(packed, torch.uint8, "packed"),
                                  _ptr(scales, torch.float32, "scales"), _stream(stream)), "pb_quantize_pack")


def pb_quantize_pack_desc(W, d, packed, scales, stream=None):
    _check(lib().pb_quantize_pack_desc(_ptr(W, torch.float32, "W"), ctypes.byref(d),
                                       _ptr(packed, torch.uint8, "packed"), _ptr(scales, torch.float32, "scales"),
                                       _stream(stream)), "pb_quantize_pack_desc")


def pb_quantize_pack_mode(W, d, quantizer, packed, scales, stream=None):
    _check(lib().pb_quantize_pack_mode(_ptr(W, torch.float32, "W"), ctypes.byref(d), quantizer,
                                       _ptr(packed, torch.uint8, "packed"), _ptr(scales, torch.float32, "scales"),
                                       _stream(stream)), "pb_quantize_pack_mode")


def pb_unpack(packed, d, q, stream=None):
    _check(lib().pb_unpack(_ptr(packed, torch.uint8, "packed"), ctypes.byref(d), _ptr(q, torch.int32, "q"),
                           _stream(stream)), "pb_unpack")


def pb_matmul(packed, scales, d, bits_used, X, batch, Y, workspace, stream=None):
    _check(lib().pb_matmul(_ptr(packed, torch.uint8, "packed"), _ptr(scales, torch.float32, "scales"),
                           ctypes.byref(d), bits_used, _ptr(X, torch.float32, "X"), batch,
                           _ptr(Y, torch.float32, "Y"), _ptr(workspace, torch.uint8, "workspace"),
                           _stream(stream)), "pb_matmul")


def pb_matmul_static(packed, scales, d, bits_used, X, batch, Y, stream=None):
    _check(lib().pb_matmul_static(_ptr(packed, torch.uint8, "packed"), _ptr(scales, torch.float32, "scales"),
                                  ctypes.byref(d), bits_used, _ptr(X, torch.float32, "X"), batch,
                                  _ptr(Y, torch.float32, "Y"), _stream(stream)), "pb_matmul_static")


def pb_matmul_bias_act(packed, scales, d, bits_used, X, batch, bias, act, Y, workspace, stream=None):
    _check(lib().pb_matmul_bias_act(_ptr(packed, torch.uint8, "packed"), _ptr(scales, torch.float32, "scales"),
                                    ctypes.byref(d), bits_used, _ptr(X, torch.float32, "X"), batch,
                                    _ptr(bias, torch.float32, "bias"), act, _ptr(Y, torch.float32, "Y"),
                                    _ptr(workspace, torch.uint8, "workspace"), _stream(stream)),
           "pb_matmul_bias_act")


def pb_matmul_acc(packed, d, bits_used, X, batch, A, workspace, stream=None):
    _check(lib().pb_matmul_acc(_ptr(packed, torch.uint8, "packed"), ctypes.byref(d), bits_used,
                               _ptr(X, torch.float32, "X"), batch, _ptr(A, torch.int64, "A"),
                               _ptr(workspace, torch.uint8, "workspace"), _stream(stream)), "pb_matmul_acc")


def pb_matmul_acc_pairs(packed, d, bits_used, X, batch, A, workspace, stream=None):
    _check(lib().pb_matmul_acc_pairs(_ptr(packed, torch.uint8, "packed"), ctypes.byref(d), bits_used,
                                     _ptr(X, torch.float32, "X"), batch, _ptr(A, torch.int64, "A"),
                                     _ptr(workspace, torch.uint8, "workspace"), _stream(stream)),
           "pb_matmul_acc_pairs")


def pb_act_prep(d, X, batch, workspace, stream=None):
    _check(lib().pb_act_prep(ctypes.byref(d), _ptr(X, torch.float32, "X"), batch,
                             _ptr(workspace, torch.uint8, "workspace"), _stream(stream)), "pb_act_prep")


def pb_matmul_prepared(packed, scales, d, bits_used, batch, Y, workspace, stream=None):
    _check(lib().pb_matmul_prepared(_ptr(packed, torch.uint8, "packed"), _ptr(scales, torch.float32, "scales"),
                                    ctypes.byref(d), bits_used, batch, _ptr(Y, torch.float32, "Y"),
                                    _ptr(workspace, torch.uint8, "workspace"), _stream(stream)),
           "pb_matmul_prepared")


def pb_fixed_point(d, X, batch, xq, workspace, stream=None):
    _check(lib().pb_fixed_point(ctypes.byref(d), _ptr(X, torch.float32, "X"), batch, _ptr(xq, torch.int32, "xq"),
                                _ptr(workspace, torch.uint8, "workspace"), _stream(stream)), "pb_fixed_point")


def pb_lstm_cell(packed, scales, d, bits_used, x_t, input_size, h_prev, c_prev, bias, h_out, c_out, batch, workspace,
                 stream=None):
    _check(lib().pb_lstm_cell(_ptr(packed, torch.uint8, "packed"), _ptr(scales, torch.float32, "scales"),
                              ctypes.byref(d), bits_used, _ptr(x_t, torch.float32, "x_t"), input_size,
                              _ptr(h_prev, torch.float32, "h_prev"), _ptr(c_prev, torch.float32, "c_prev"),
                              _ptr(bias, torch.float32, "bias"), _ptr(h_out, torch.float32, "h_out"),
                              _ptr(c_out, torch.float32, "c_out"), batch,
                              _ptr(workspace, torch.uint8, "workspace"), _stream(stream)), "pb_lstm_cell")


class PackedLinear:
    """Convenience holder: one quantized, packed weight matrix with its scales and a workspace."""

    def __init__(self, W: torch.Tensor, bits: int, max_batch: int = 1, frac_bits: int = 16, act_bits: int = 32,
                 layout: int | None = None, quantizer: int = PB_QUANT_SYMMETRIC):
        assert W.is_cuda and W.dtype == torch.float32 and W.dim() == 2
        W = W.contiguous()
        self.rows, self.cols = W.shape
        self.bits = bits
        if layout is None:
            self.desc = pb_desc_init(self.rows, self.cols, bits, frac_bits, act_bits)
        else:
            self.desc = pb_desc_init_layout(self.rows, self.cols, bits, layout, frac_bits, act_bits)
        self.packed = alloc_packed(self.desc, W.device)
        self.scales = torch.empty(max(bits, 4), dtype=torch.float32, device=W.device)
        self.max_batch = max_batch
        self.workspace = alloc_workspace(self.desc, max_batch, W.device)
        pb_quantize_pack_mode(W, self.desc, quantizer, self.packed, self.scales)

    def __call__(self, X: torch.Tensor, bits_used: int | None = None, out: torch.Tensor | None = None):
        X = X.reshape(-1, self.cols)
        batch = X.shape[0]
        assert batch <= self.max_batch
        if out is None:
            out = torch.empty((batch, self.rows), dtype=torch.float32, device=X.device)
        pb_matmul(self.packed, self.scales, self.desc, bits_used or self.bits, X, batch, out, self.workspace)
        return out

    def acc(self, X: torch.Tensor, bits_used: int | None = None):
        X = X.reshape(-1, self.cols)
        batch = X.shape[0]
        m = bits_used or self.bits
        A = torch.empty((m, batch, self.rows), dtype=torch.int64, device=X.device)
        pb_matmul_acc(self.packed, self.desc, m, X, batch, A, self.workspace)
        return A

    def acc_pairs(self, X: torch.Tensor, bits_used: int | None = None):
        X = X.reshape(-1, self.cols)
        batch = X.shape[0]
        m = bits_used or self.bits
        A = torch.empty(((m + 1) // 2, batch, self.rows), dtype=torch.int64, device=X.device)
        pb_matmul_acc_pairs(self.packed, self.desc, m, X, batch, A, self.workspace)
        return A

    def unpack(self):
        q = torch.empty((self.rows, self.cols), dtype=torch.int32, device=self.packed.device)
        pb_unpack(self.packed, self.desc, q)
        return q
