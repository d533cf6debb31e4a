"""ctypes front end of the MXInt CPU oracle (``mx_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

Nothing in the GPU library imports this module; only the tests, the smoke check
and the CPU-baseline leg of the benchmark do.  Every function here only
marshals numpy arrays into the plain C routines of the C file, which holds the
arithmetic of the quantizers, the bit packing, the width cast and the product
(and the statement of what the paper fixes and what is a reading of it).  Three
compositions of those routines are written here in numpy: ``linear_q`` (product,
bias, output quantizer), ``attention`` (the four steps of an MXInt attention
head) and the regrouping of rows for two-row blocks (``block_rows``).

Format arguments follow Section 4.1 of the paper: ``block`` elements share one
``e``-bit exponent; ``w`` is the stored width of an element, i.e. the paper's
mantissa width m plus the sign bit (Eq. 1).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mx_oracle.c")
_LIB = os.path.join(_HERE, "libmx_oracle.so")

RNE = 0
RTZ = 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, no intrinsics)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, p = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.mxo_quantize.argtypes = [p, i64, i64, i64, i32, i32, i32, i32, p, p]
        lib.mxo_quantize_axis0.argtypes = [p, i64, i64, i64, i32, i32, i32, i32, p, p]
        lib.mxo_dequantize.argtypes = [p, p, i64, i64, i32, i32, i32, p]
        lib.mxo_pack_bits.argtypes = [p, i64, i64, i32, p]
        lib.mxo_unpack_bits.argtypes = [p, i64, i64, i32, p]
        lib.mxo_gemm.argtypes = [p, p, i32, p, p, i32, i64, i64, i64, i32, i32, i64, i64, p, p]
        lib.mxo_set_threads.argtypes = [i32]
        lib.mxo_cast.argtypes = [p, p, i64, i64, i32, i32, i32, i32, i32, i32, p, p]
        lib.mxo_quantize_minifloat.argtypes = [p, i64, i64, i64, i32, i32, i32, i32, p, p]
        lib.mxo_dequantize_minifloat.argtypes = [p, p, i64, i64, i32, i32, i32, p]
        for f in (lib.mxo_quantize, lib.mxo_quantize_axis0, lib.mxo_dequantize, lib.mxo_pack_bits,
                  lib.mxo_unpack_bits, lib.mxo_gemm, lib.mxo_set_threads, lib.mxo_cast,
                  lib.mxo_quantize_minifloat, lib.mxo_dequantize_minifloat):
            f.restype = i32
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc == 1:
        raise ValueError("%s: bad argument" % what)
    if rc == 2:
        raise ValueError("%s: input holds a NaN or an infinity" % what)
    if rc != 0:
        raise RuntimeError("%s: status %d" % (what, rc))


def set_threads(n: int) -> int:
    """Set the number of OpenMP threads the row loops use; returns the count in force."""
    return int(_load().mxo_set_threads(int(n)))


def quantize(x: np.ndarray, block: int, w: int, e: int = 8, rounding: int = RNE,
             axis: int = 1, block_rows: int = 1) -> Tuple[np.ndarray, np.ndarray]:
    """Quantize a 2-D float32 array to MXInt.

    axis=1: blocks along each row; returns q int8 [rows, cols], exps uint8 [rows, cols/block].
    axis=0: blocks down each column; returns the quantization of x.T:
            q int8 [cols, rows], exps uint8 [cols, rows/block].
    block_rows=R > 1 (axis 1 only): the paper's two-dimensional block shape (block, R) of
            Section 4.1, e.g. MXInt((16,2),8,7): R adjacent rows x block columns share one
            exponent.  A block is just a set of R*block elements, so the rows are regrouped and
            the one-dimensional routine is applied; exps is uint8 [rows/R, cols/block].
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert x.ndim == 2
    rows, cols = x.shape
    lib = _load()
    if block_rows != 1:
        if axis != 1 or block_rows < 1 or rows % block_rows or block < 1 or cols % block:
            raise ValueError("two-dimensional blocks need axis 1, rows % block_rows == 0, cols % block == 0")
        R, nb = block_rows, cols // block
        # [rows/R, R, nb, block] -> [rows/R, nb, R, block]: every block's elements become one run
        xr = np.ascontiguousarray(x.reshape(rows // R, R, nb, block).transpose(0, 2, 1, 3)).reshape(rows // R, nb * R * block)
        qr, ex = quantize(xr, R * block, w, e, rounding)
        q = np.ascontiguousarray(qr.reshape(rows // R, nb, R, block).transpose(0, 2, 1, 3)).reshape(rows, cols)
        return q, ex
    if axis == 1:
        if block < 1 or cols % block:
            raise ValueError("cols must be a multiple of block")
        q = np.empty((rows, cols), np.int8)
        ex = np.empty((rows, cols // block), np.uint8)
        rc = lib.mxo_quantize(_ptr(x), rows, cols, cols, block, e, w, rounding, _ptr(q), _ptr(ex))
    else:
        if block < 1 or rows % block:
            raise ValueError("rows must be a multiple of block")
        q = np.empty((cols, rows), np.int8)
        ex = np.empty((cols, rows // block), np.uint8)
        rc = lib.mxo_quantize_axis0(_ptr(x), rows, cols, cols, block, e, w, rounding, _ptr(q), _ptr(ex))
    _check(rc, "quantize")
    return q, ex


def row_exps(exps: np.ndarray, block_rows: int) -> np.ndarray:
    """Exponent bytes of a two-dimensional-block tensor [rows/R, nblk] spelled out per row [rows, nblk]
    (the form dequantize, gemm and cast take)."""
    return np.repeat(np.ascontiguousarray(exps, dtype=np.uint8), block_rows, axis=0)


def dequantize(q: np.ndarray, exps: np.ndarray, block: int, w: int, e: int = 8) -> np.ndarray:
    """Exact values of an MXInt tensor, as float64 [rows, cols]."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    exps = np.ascontiguousarray(exps, dtype=np.uint8)
    rows, cols = q.shape
    assert exps.shape == (rows, cols // block)
    y = np.empty((rows, cols), np.float64)
    _check(_load().mxo_dequantize(_ptr(q), _ptr(exps), rows, cols, block, e, w, _ptr(y)), "dequantize")
    return y


def cast(q: np.ndarray, exps: np.ndarray, block: int, ws: int, wd: int, es: int = 8, ed: int = 8,
         rounding: int = RNE, block_rows: int = 1) -> Tuple[np.ndarray, np.ndarray]:
    """MXInt (block, es, ws) -> MXInt (block, ed, wd) in integer arithmetic: mantissa extension or
    rounding shift plus exponent renormalisation (Section 4, mixed-precision paragraph).
    q int8 [rows, cols], exps uint8 [rows/block_rows, cols/block]; returns the same shapes.
    Two-dimensional blocks are regrouped into runs, as in quantize."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    exps = np.ascontiguousarray(exps, dtype=np.uint8)
    rows, cols = q.shape
    if block_rows != 1:
        R, nb = block_rows, cols // block
        assert rows % R == 0 and exps.shape == (rows // R, nb)
        qr = np.ascontiguousarray(q.reshape(rows // R, R, nb, block).transpose(0, 2, 1, 3)).reshape(rows // R, nb * R * block)
        q2, e2 = cast(qr, exps, R * block, ws, wd, es, ed, rounding)
        return np.ascontiguousarray(q2.reshape(rows // R, nb, R, block).transpose(0, 2, 1, 3)).reshape(rows, cols), e2
    assert exps.shape == (rows, cols // block)
    q2 = np.empty((rows, cols), np.int8)
    e2 = np.empty((rows, cols // block), np.uint8)
    _check(_load().mxo_cast(_ptr(q), _ptr(exps), rows, cols, block, es, ws, ed, wd, rounding, _ptr(q2),
                            _ptr(e2)), "cast")
    return q2, e2


def pack_bits(q: np.ndarray, w: int) -> np.ndarray:
    """Signed mantissas int8 [rows, cols] -> uint8 [rows, cols*w/8] little-endian bit stream."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    rows, cols = q.shape
    out = np.empty((rows, cols * w // 8), np.uint8)
    _check(_load().mxo_pack_bits(_ptr(q), rows, cols, w, _ptr(out)), "pack_bits")
    return out


def unpack_bits(packed: np.ndarray, cols: int, w: int) -> np.ndarray:
    """Inverse of pack_bits."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    rows = packed.shape[0]
    assert packed.shape[1] == cols * w // 8
    q = np.empty((rows, cols), np.int8)
    _check(_load().mxo_unpack_bits(_ptr(packed), rows, cols, w, _ptr(q)), "unpack_bits")
    return q


def gemm(qa: np.ndarray, ea: np.ndarray, wa: int, qb: np.ndarray, eb: np.ndarray, wb: int,
         block: int, e: int = 8, rows: Optional[Tuple[int, int]] = None,
         want_mag: bool = False):
    """Y[m,n] = sum over K-blocks of (exact integer block dot) * 2^(sum of the two block exponents).

    qa [M,K], ea [M,K/block]; qb [N,K] (the right operand stored row-per-output-column), eb [N,K/block].
    Returns float64 [M,N] (rows outside ``rows=(begin,end)`` are left as NaN), and with
    want_mag also sum_b |term_b|.
    """
    qa = np.ascontiguousarray(qa, dtype=np.int8)
    qb = np.ascontiguousarray(qb, dtype=np.int8)
    ea = np.ascontiguousarray(ea, dtype=np.uint8)
    eb = np.ascontiguousarray(eb, dtype=np.uint8)
    M, K = qa.shape
    N, K2 = qb.shape
    assert K == K2 and ea.shape == (M, K // block) and eb.shape == (N, K // block)
    m0, m1 = (0, M) if rows is None else rows
    y = np.full((M, N), np.nan, np.float64)
    mag = np.full((M, N), np.nan, np.float64) if want_mag else None
    rc = _load().mxo_gemm(_ptr(qa), _ptr(ea), wa, _ptr(qb), _ptr(eb), wb, M, N, K, block, e, m0, m1,
                          _ptr(y), _ptr(mag) if want_mag else None)
    _check(rc, "gemm")
    return (y, mag) if want_mag else y


def linear(x: np.ndarray, wt: np.ndarray, block: int, wx: int, ww: int, e: int = 8,
           rounding: int = RNE, want_mag: bool = False):
    """Quantize x [M,K] and wt [N,K] along K, then the MXInt product: the emulated linear layer
    of Section 3.2 without output re-quantization."""
    qa, ea = quantize(x, block, wx, e, rounding)
    qb, eb = quantize(wt, block, ww, e, rounding)
    return gemm(qa, ea, wx, qb, eb, ww, block, e, want_mag=want_mag)


def linear_q(x: np.ndarray, wt: np.ndarray, bias: Optional[np.ndarray], block: int, wx: int, ww: int, wbias: int,
             wo: int, e: int = 8, rounding: int = RNE, block_rows: int = 1):
    """The emulated linear layer of Section 3.2 in full (the LinearOp of Fig. 2b): quantize x [M,K], the
    weights wt [N,K] and the bias [N] to MXInt, take the MXInt product, add the bias, and quantize the
    result (held in fp32, the emulator's working precision) to the output format, blocks along N.

    Returns (q_out int8 [M,N], exps_out uint8 [M/block_rows, N/block], y float64 [M,N] before the output
    quantizer, mag float64 [M,N] = sum_b |term_b| + |bias|)."""
    qa, ea = quantize(x, block, wx, e, rounding, block_rows=block_rows)
    qb, eb = quantize(wt, block, ww, e, rounding, block_rows=block_rows)
    y, mag = gemm(qa, row_exps(ea, block_rows), wx, qb, row_exps(eb, block_rows), ww, block, e, want_mag=True)
    if bias is not None:
        bq, be = quantize(np.asarray(bias, np.float32).reshape(1, -1), block, wbias, e, rounding)
        bv = dequantize(bq, be, block, wbias, e)
        y = y + bv
        mag = mag + np.abs(bv)
    qo, eo = quantize(y.astype(np.float32), block, wo, e, rounding, block_rows=block_rows)
    return qo, eo, y, mag


def attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, block: int, wq: int, wk: int, wp: int, wv: int,
              scale: float, e: int = 8, rounding: int = RNE, rows: Optional[Tuple[int, int]] = None,
              block_rows: int = 1, e_pv: Optional[int] = None):
    """One head of attention with every matrix product taken in MXInt (Fig. 1: the two products of the
    attention layer have both operands quantized; Section 3.2: an emulated operator quantizes its inputs
    and computes on the quantized values; softmax itself stays in floating point).

    Q [Sq,D], K [Sk,D], V [Sk,D] float32.  Steps, in the order of the definition:
      1. Q and K are quantized in blocks along D;  S = MXInt product Q K^T                       [Sq,Sk]
      2. P = softmax(scale * S) along the keys, in float64, then held as float32 (the quantizer's input type)
      3. P is quantized in blocks along the keys, V in blocks along the keys (down its columns)
      4. O = MXInt product P V                                                                   [Sq,D]
    Returns O float64 [Sq,D] and a dict with the intermediate values the tests derive tolerances from:
    S, S_mag (sum_b |term_b| of step 1), P (float64), pq/pe and vq/ve (the quantized operands of step 4)
    and O_mag.  rows=(begin,end) restricts the query rows that are computed (others are NaN).
    block_rows=2: every tensor in the paper's two-dimensional block shape (block, 2) (Section 3, the MASE IR example; Section 4.1) -- two
    neighbouring rows of the matrix that is quantized share their exponents: two queries (Q, P), two keys
    (K), two columns of V (the rows of V^T).  pe and ve then hold one exponent row per matrix row (each
    shared row repeated), as the product takes them.
    e_pv: exponent width of P and V, the operands of the second product (default: e, the width of Q and K;
    Section 4.1 lets the exponent width be chosen per tensor even though the paper then fixes 8 for all)."""
    if e_pv is None:
        e_pv = e
    Q = np.ascontiguousarray(Q, np.float32)
    K = np.ascontiguousarray(K, np.float32)
    V = np.ascontiguousarray(V, np.float32)
    r0, r1 = (0, Q.shape[0]) if rows is None else rows
    R = block_rows
    if R != 1 and (r0 % R or r1 % R):
        raise ValueError("the row window must hold whole row groups")
    qq, qe = quantize(Q[r0:r1], block, wq, e, rounding, block_rows=R)
    kq, ke = quantize(K, block, wk, e, rounding, block_rows=R)
    S, s_mag = gemm(qq, row_exps(qe, R), wq, kq, row_exps(ke, R), wk, block, e, want_mag=True)
    Z = np.float64(scale) * S
    Z = Z - Z.max(axis=1, keepdims=True)
    P = np.exp(Z)
    P = P / P.sum(axis=1, keepdims=True)
    pq, pe = quantize(P.astype(np.float32), block, wp, e_pv, rounding, block_rows=R)
    if R == 1:
        vq, ve = quantize(V, block, wv, e_pv, rounding, axis=0)   # the quantization of V^T: [D, Sk]
    else:
        vq, ve = quantize(np.ascontiguousarray(V.T), block, wv, e_pv, rounding, block_rows=R)
    pe, ve = row_exps(pe, R), row_exps(ve, R)
    Osub, o_mag = gemm(pq, pe, wp, vq, ve, wv, block, e_pv, want_mag=True)
    O = np.full((Q.shape[0], V.shape[1]), np.nan, np.float64)
    O[r0:r1] = Osub
    return O, {"S": S, "S_mag": s_mag, "P": P, "pq": pq, "pe": pe, "vq": vq, "ve": ve, "O_mag": o_mag,
               "rows": (r0, r1), "block_rows": R}


def quantize_minifloat(x: np.ndarray, block: int, e: int, m: int, rounding: int = RNE) -> Tuple[np.ndarray, np.ndarray]:
    """The paper's other block formats (Section 2): Block Minifloat BMF(block, e, m) -- sign, e exponent bits,
    m mantissa bits per element, the exponent bias shared by the block -- and, with m = 0, Block Logarithm
    (powers of two).  Returns codes uint8 [rows, cols] (sign << (e+m) | c << m | f) and the shared byte
    (top exponent + 127) uint8 [rows, cols/block]; the bit-level reading is stated in the C file."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert x.ndim == 2
    rows, cols = x.shape
    if block < 1 or cols % block:
        raise ValueError("cols must be a multiple of block")
    codes = np.empty((rows, cols), np.uint8)
    shared = np.empty((rows, cols // block), np.uint8)
    _check(_load().mxo_quantize_minifloat(_ptr(x), rows, cols, cols, block, e, m, rounding, _ptr(codes), _ptr(shared)),
           "quantize_minifloat")
    return codes, shared


def dequantize_minifloat(codes: np.ndarray, shared: np.ndarray, block: int, e: int, m: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    shared = np.ascontiguousarray(shared, dtype=np.uint8)
    rows, cols = codes.shape
    y = np.empty((rows, cols), np.float64)
    _check(_load().mxo_dequantize_minifloat(_ptr(codes), _ptr(shared), rows, cols, block, e, m, _ptr(y)),
           "dequantize_minifloat")
    return y
