"""ctypes binding of ``libmx.so`` -- argument marshalling only.

Every function here has the name of the C entry point it calls (``include/mx.h``) and passes
device pointers of torch tensors plus the current HIP stream; torch supplies device memory and
streams, nothing else.  There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmx.so")

MX_RNE, MX_RTZ = 0, 1
MX_OK, MX_ERR_BAD_ARG, MX_ERR_UNSUPPORTED, MX_ERR_DEVICE = 0, 1, 2, 3
MX_LAYOUT_FRAGMENT = 0
MX_LAYOUT_MATRIX = 1

EXPORTS = ("mx_version", "mx_status_string", "mx_mant_bytes", "mx_exps_bytes", "mx_quantize", "mx_check_finite",
           "mx_dequantize", "mx_cast", "mx_packed_bytes", "mx_pack", "mx_quantize_pack", "mx_quantize_pack_axis0", "mx_unpack",
           "mx_gemm",
           "mx_gemm_q", "mx_attention", "mx_linear", "mx_linear_workspace_bytes", "mx_linear_static_workspace",
           "mx_linear_static_workspace_max", "mx_quantize_minifloat",
           "mx_dequantize_minifloat")


class mx_format(ctypes.Structure):
    """Mirror of the C struct: block, exp_bits, mant_bits (stored bits incl. sign), rounding, block_rows."""
    _fields_ = [("block", ctypes.c_int32), ("exp_bits", ctypes.c_int32),
                ("mant_bits", ctypes.c_int32), ("rounding", ctypes.c_int32), ("block_rows", ctypes.c_int32)]

    def __repr__(self):
        return "mx_format(block=%d, exp_bits=%d, mant_bits=%d, rounding=%d, block_rows=%d)" % (
            self.block, self.exp_bits, self.mant_bits, self.rounding, self.block_rows)


def fmt(block: int, mant_bits: int, exp_bits: int = 8, rounding: int = MX_RNE, block_rows: int = 1) -> mx_format:
    return mx_format(block, exp_bits, mant_bits, rounding, block_rows)


class mx_minifloat_format(ctypes.Structure):
    """Mirror of the C struct of the Block Minifloat / Block Logarithm formats: block, exp_bits, mant_bits, rounding."""
    _fields_ = [("block", ctypes.c_int32), ("exp_bits", ctypes.c_int32), ("mant_bits", ctypes.c_int32),
                ("rounding", ctypes.c_int32)]


class MxError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s: %s" % (what, status_string(status)))


_lib = None


def load() -> ctypes.CDLL:
    """Load the built library; raises if it is missing (build it with ``python -m paper_2307_15517_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build it with `python -m paper_2307_15517_amd.build`" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    i32, i64, vp, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    lib.mx_version.argtypes, lib.mx_version.restype = [], i32
    lib.mx_status_string.argtypes, lib.mx_status_string.restype = [i32], ctypes.c_char_p
    lib.mx_mant_bytes.argtypes, lib.mx_mant_bytes.restype = [i64, i64, i64, mx_format], sz
    lib.mx_exps_bytes.argtypes, lib.mx_exps_bytes.restype = [i64, i64, i64, mx_format], sz
    lib.mx_quantize.argtypes = [vp, i64, i64, i64, i64, i64, i32, mx_format, vp, vp, vp]
    lib.mx_dequantize.argtypes = [vp, vp, i64, i64, i64, mx_format, vp, vp]
    lib.mx_check_finite.argtypes, lib.mx_check_finite.restype = [vp, i64, i64, i64, i64, i64, vp, vp], i32
    lib.mx_cast.argtypes = [vp, vp, i64, i64, i64, mx_format, mx_format, vp, vp, vp]
    lib.mx_packed_bytes.argtypes, lib.mx_packed_bytes.restype = [i64, i64, i64, mx_format, i32], sz
    lib.mx_pack.argtypes = [vp, vp, i64, i64, i64, mx_format, i32, vp, vp]
    lib.mx_quantize_pack.argtypes = [vp, i64, i64, i64, i64, i64, mx_format, i32, vp, vp]
    lib.mx_quantize_pack_axis0.argtypes = [vp, i64, i64, i64, i64, i64, mx_format, i32, vp, vp]
    lib.mx_unpack.argtypes = [vp, i64, i64, i64, mx_format, i32, vp, vp, vp]
    lib.mx_gemm.argtypes = [i64, i64, i64, i64, vp, mx_format, vp, mx_format, i32, vp, i64, i64, vp]
    lib.mx_gemm_q.argtypes = [i64, i64, i64, i64, vp, mx_format, vp, mx_format, i32, vp, vp, mx_format, mx_format, vp, vp]
    lib.mx_attention.argtypes = [i64, i64, i64, i64, vp, mx_format, vp, mx_format, vp, mx_format, mx_format,
                                 ctypes.c_float, i32, vp, i64, i64, vp]
    lib.mx_quantize_minifloat.argtypes = [vp, i64, i64, i64, i64, i64, mx_minifloat_format, vp, vp, vp]
    lib.mx_dequantize_minifloat.argtypes = [vp, vp, i64, i64, i64, mx_minifloat_format, vp, vp]
    lib.mx_linear.argtypes = [vp, i64, i64, i64, mx_format, vp, vp, i64, mx_format, i32, vp, i64, vp]
    lib.mx_linear_workspace_bytes.argtypes = [i64, i64, i64, mx_format, mx_format, i32]
    lib.mx_linear_workspace_bytes.restype = sz
    lib.mx_linear_static_workspace.argtypes = [vp, i64, i64, i64, mx_format, vp, i64, mx_format, i32, vp, i64, vp]
    lib.mx_linear_static_workspace.restype = i32
    lib.mx_linear_static_workspace_max.argtypes, lib.mx_linear_static_workspace_max.restype = [], sz
    for name in ("mx_quantize", "mx_dequantize", "mx_cast", "mx_pack", "mx_quantize_pack", "mx_quantize_pack_axis0",
                 "mx_unpack", "mx_gemm",
                 "mx_gemm_q", "mx_attention", "mx_linear", "mx_quantize_minifloat", "mx_dequantize_minifloat"):
        getattr(lib, name).restype = i32
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().mx_status_string(int(status)).decode()


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


def _p(t) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _raise(status: int, what: str):
    if status != MX_OK:
        raise MxError(status, what)


# ---- the entry points, same names as in include/mx.h ---------------------------------------------
def mx_version() -> int:
    return int(load().mx_version())


def mx_mant_bytes(batch: int, rows: int, cols: int, f: mx_format) -> int:
    return int(load().mx_mant_bytes(batch, rows, cols, f))


def mx_exps_bytes(batch: int, rows: int, cols: int, f: mx_format) -> int:
    return int(load().mx_exps_bytes(batch, rows, cols, f))


def mx_packed_bytes(batch: int, rows: int, cols: int, f: mx_format, layout: int = MX_LAYOUT_FRAGMENT) -> int:
    return int(load().mx_packed_bytes(batch, rows, cols, f, layout))


def mx_quantize(x, batch, rows, cols, row_stride, batch_stride, axis, f, mant, exps, stream=None,
                check: bool = True) -> int:
    s = load().mx_quantize(_p(x), batch, rows, cols, row_stride, batch_stride, axis, f, _p(mant),
                           _p(exps), _stream(stream))
    if check:
        _raise(s, "mx_quantize")
    return s


def mx_check_finite(x, batch, rows, cols, row_stride, batch_stride, flag, stream=None) -> int:
    """The status itself is the answer (MX_OK: all finite, MX_ERR_BAD_ARG: a NaN or an infinity, or a bad argument)."""
    return load().mx_check_finite(_p(x), batch, rows, cols, row_stride, batch_stride, _p(flag), _stream(stream))


def mx_dequantize(mant, exps, batch, rows, cols, f, y, stream=None, check: bool = True) -> int:
    s = load().mx_dequantize(_p(mant), _p(exps), batch, rows, cols, f, _p(y), _stream(stream))
    if check:
        _raise(s, "mx_dequantize")
    return s


def mx_cast(mant, exps, batch, rows, cols, fs, fd, mant_out, exps_out, stream=None, check: bool = True) -> int:
    s = load().mx_cast(_p(mant), _p(exps), batch, rows, cols, fs, fd, _p(mant_out), _p(exps_out), _stream(stream))
    if check:
        _raise(s, "mx_cast")
    return s


def mx_pack(mant, exps, batch, rows, cols, f, layout, packed, stream=None, check: bool = True) -> int:
    s = load().mx_pack(_p(mant), _p(exps), batch, rows, cols, f, layout, _p(packed), _stream(stream))
    if check:
        _raise(s, "mx_pack")
    return s


def mx_quantize_pack(x, batch, rows, cols, row_stride, batch_stride, f, layout, packed, stream=None,
                     check: bool = True) -> int:
    s = load().mx_quantize_pack(_p(x), batch, rows, cols, row_stride, batch_stride, f, layout, _p(packed),
                                _stream(stream))
    if check:
        _raise(s, "mx_quantize_pack")
    return s


def mx_quantize_pack_axis0(x, batch, rows, cols, row_stride, batch_stride, f, layout, packed, stream=None,
                           check: bool = True) -> int:
    s = load().mx_quantize_pack_axis0(_p(x), batch, rows, cols, row_stride, batch_stride, f, layout, _p(packed),
                                      _stream(stream))
    if check:
        _raise(s, "mx_quantize_pack_axis0")
    return s


def mx_unpack(packed, batch, rows, cols, f, layout, mant, exps, stream=None, check: bool = True) -> int:
    s = load().mx_unpack(_p(packed), batch, rows, cols, f, layout, _p(mant), _p(exps), _stream(stream))
    if check:
        _raise(s, "mx_unpack")
    return s


def mx_gemm(batch, M, N, K, A_packed, fa, B_packed, fb, layout, Y, ldy, batch_stride_y, stream=None,
            check: bool = True) -> int:
    s = load().mx_gemm(batch, M, N, K, _p(A_packed), fa, _p(B_packed), fb, layout, _p(Y), ldy,
                       batch_stride_y, _stream(stream))
    if check:
        _raise(s, "mx_gemm")
    return s


def mx_gemm_q(batch, M, N, K, A_packed, fa, B_packed, fb, layout, bias_mant, bias_exps, fbias, fo, out_packed,
              stream=None, check: bool = True) -> int:
    s = load().mx_gemm_q(batch, M, N, K, _p(A_packed), fa, _p(B_packed), fb, layout, _p(bias_mant), _p(bias_exps),
                         fbias, fo, _p(out_packed), _stream(stream))
    if check:
        _raise(s, "mx_gemm_q")
    return s


def mx_attention(batch, Sq, Sk, D, Q_packed, fq, K_packed, fk, Vt_packed, fv, fp, scale, layout, O, ldo,
                 o_batch_stride, stream=None, check: bool = True) -> int:
    s = load().mx_attention(batch, Sq, Sk, D, _p(Q_packed), fq, _p(K_packed), fk, _p(Vt_packed), fv, fp,
                            float(scale), layout, _p(O), ldo, o_batch_stride, _stream(stream))
    if check:
        _raise(s, "mx_attention")
    return s


def mx_quantize_minifloat(x, batch, rows, cols, row_stride, batch_stride, f, codes, shared, stream=None,
                          check: bool = True) -> int:
    s = load().mx_quantize_minifloat(_p(x), batch, rows, cols, row_stride, batch_stride, f, _p(codes), _p(shared),
                                     _stream(stream))
    if check:
        _raise(s, "mx_quantize_minifloat")
    return s


def mx_dequantize_minifloat(codes, shared, batch, rows, cols, f, y, stream=None, check: bool = True) -> int:
    s = load().mx_dequantize_minifloat(_p(codes), _p(shared), batch, rows, cols, f, _p(y), _stream(stream))
    if check:
        _raise(s, "mx_dequantize_minifloat")
    return s


def mx_linear_workspace_bytes(M: int, K: int, N: int, fx: mx_format, fb: mx_format,
                              layout: int = MX_LAYOUT_FRAGMENT) -> int:
    return int(load().mx_linear_workspace_bytes(M, K, N, fx, fb, layout))


def mx_linear(x, M, K, row_stride, fx, workspace, B_packed, N, fb, layout, Y, ldy, stream=None,
              check: bool = True) -> int:
    s = load().mx_linear(_p(x), M, K, row_stride, fx, _p(workspace), _p(B_packed), N, fb, layout, _p(Y),
                         ldy, _stream(stream))
    if check:
        _raise(s, "mx_linear")
    return s


def mx_linear_static_workspace(x, M, K, row_stride, fx, B_packed, N, fb, layout, Y, ldy, stream=None,
                               check: bool = True) -> int:
    s = load().mx_linear_static_workspace(_p(x), M, K, row_stride, fx, _p(B_packed), N, fb, layout, _p(Y), ldy,
                                          _stream(stream))
    if check:
        _raise(s, "mx_linear_static_workspace")
    return s


def mx_linear_static_workspace_max() -> int:
    return int(load().mx_linear_static_workspace_max())


def bound(name: str, *args, stream=None):
    """Marshal the arguments of entry point ``name`` once and return a zero-argument callable that
    issues exactly that call again (status checked).  For loops that launch the same call many times:
    per-call marshalling costs several microseconds, more than a small kernel runs.  The tensors must
    stay alive, and the stream current at binding time is the one used."""
    fn = getattr(load(), name)
    cargs = []
    for a in args:
        if a is None or isinstance(a, torch.Tensor):
            cargs.append(_p(a))
        else:
            cargs.append(a)
    cargs.append(_stream(stream))
    cargs = tuple(cargs)

    def call():
        s = fn(*cargs)
        if s != MX_OK:
            raise MxError(s, name)
    return call


# ---- conveniences that only allocate outputs with torch and call the entry points above -----------
def check_finite(x: torch.Tensor) -> bool:
    """True when every element of the float32 CUDA tensor [rows, cols] or [batch, rows, cols] is finite."""
    assert x.is_cuda and x.dtype == torch.float32 and x.stride(-1) == 1
    if x.dim() == 2:
        batch, (rows, cols), bs = 1, x.shape, 0
    else:
        batch, rows, cols = x.shape
        bs = x.stride(0)
    flag = torch.empty(1, dtype=torch.int32, device=x.device)
    s = mx_check_finite(x, batch, rows, cols, x.stride(-2), bs, flag)
    if s not in (MX_OK, MX_ERR_BAD_ARG):
        _raise(s, "mx_check_finite")
    return s == MX_OK


def quantize(x: torch.Tensor, f: mx_format, axis: int = 1) -> Tuple[torch.Tensor, torch.Tensor]:
    """x: float32 CUDA tensor [rows, cols] or [batch, rows, cols] with contiguous columns."""
    assert x.is_cuda and x.dtype == torch.float32 and x.stride(-1) == 1
    if x.dim() == 2:
        batch, (rows, cols), bs = 1, x.shape, 0
    else:
        batch, rows, cols = x.shape
        bs = x.stride(0)
    orows, ocols = (rows, cols) if axis == 1 else (cols, rows)
    mant = torch.empty(mx_mant_bytes(batch, orows, ocols, f), dtype=torch.uint8, device=x.device)
    exps = torch.empty(mx_exps_bytes(batch, orows, ocols, f), dtype=torch.uint8, device=x.device)
    mx_quantize(x, batch, rows, cols, x.stride(-2), bs, axis, f, mant, exps)
    return mant, exps


def dequantize(mant: torch.Tensor, exps: torch.Tensor, batch: int, rows: int, cols: int,
               f: mx_format) -> torch.Tensor:
    y = torch.empty((batch, rows, cols), dtype=torch.float32, device=mant.device)
    mx_dequantize(mant, exps, batch, rows, cols, f, y)
    return y


def cast(mant: torch.Tensor, exps: torch.Tensor, batch: int, rows: int, cols: int, fs: mx_format,
         fd: mx_format) -> Tuple[torch.Tensor, torch.Tensor]:
    """Canonical form in fs -> canonical form in fd (same block size), in integer arithmetic."""
    mant_out = torch.empty(mx_mant_bytes(batch, rows, cols, fd), dtype=torch.uint8, device=mant.device)
    exps_out = torch.empty(mx_exps_bytes(batch, rows, cols, fd), dtype=torch.uint8, device=mant.device)
    mx_cast(mant, exps, batch, rows, cols, fs, fd, mant_out, exps_out)
    return mant_out, exps_out


def pack(mant: torch.Tensor, exps: torch.Tensor, batch: int, rows: int, cols: int, f: mx_format,
         layout: int = MX_LAYOUT_FRAGMENT) -> torch.Tensor:
    packed = torch.empty(max(1, mx_packed_bytes(batch, rows, cols, f, layout)), dtype=torch.uint8,
                         device=mant.device)
    mx_pack(mant, exps, batch, rows, cols, f, layout, packed)
    return packed


def quantize_pack(x: torch.Tensor, f: mx_format, layout: int = MX_LAYOUT_FRAGMENT) -> torch.Tensor:
    """fp32 [rows, cols] or [batch, rows, cols] -> packed operand in one pass."""
    assert x.is_cuda and x.dtype == torch.float32 and x.stride(-1) == 1
    if x.dim() == 2:
        batch, (rows, cols), bs = 1, x.shape, 0
    else:
        batch, rows, cols = x.shape
        bs = x.stride(0)
    packed = torch.empty(max(1, mx_packed_bytes(batch, rows, cols, f, layout)), dtype=torch.uint8, device=x.device)
    mx_quantize_pack(x, batch, rows, cols, x.stride(-2), bs, f, layout, packed)
    return packed


def unpack(packed: torch.Tensor, batch: int, rows: int, cols: int, f: mx_format,
           layout: int = MX_LAYOUT_FRAGMENT) -> Tuple[torch.Tensor, torch.Tensor]:
    mant = torch.empty(mx_mant_bytes(batch, rows, cols, f), dtype=torch.uint8, device=packed.device)
    exps = torch.empty(mx_exps_bytes(batch, rows, cols, f), dtype=torch.uint8, device=packed.device)
    mx_unpack(packed, batch, rows, cols, f, layout, mant, exps)
    return mant, exps


def linear_workspace(M: int, K: int, N: int, fx: mx_format, fb: mx_format, device) -> torch.Tensor:
    """A zero-filled workspace for mx_linear (the arrival counters at its start must be zero before the first call)."""
    return torch.zeros(max(1, mx_linear_workspace_bytes(M, K, N, fx, fb)), dtype=torch.uint8, device=device)


def gemm(A_packed: torch.Tensor, fa: mx_format, B_packed: torch.Tensor, fb: mx_format, M: int, N: int,
         K: int, batch: int = 1, layout: int = MX_LAYOUT_FRAGMENT,
         out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if out is None:
        out = torch.empty((batch, M, N), dtype=torch.float32, device=A_packed.device)
    mx_gemm(batch, M, N, K, A_packed, fa, B_packed, fb, layout, out, N, M * N)
    return out
