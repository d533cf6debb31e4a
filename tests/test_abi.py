"""Host-side checks of the C-ABI library: it loads, exports what include/mx.h declares, does the
size accounting of the format, and rejects bad arguments before any launch.  No GPU needed."""
import ctypes
import os
import re

import pytest

from paper_2307_15517_amd import mx

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(mx.LIB_PATH):
        from paper_2307_15517_amd import build
        build.build(verbose=False)
    return mx.load()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "mx.h")).read()
    declared = re.findall(r"MX_API\s+[\w\s\*]+?\b(mx_\w+)\s*\(", header)
    assert set(declared) == set(mx.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert mx.mx_version() >= 100
    assert mx.status_string(mx.MX_OK) == "ok" and "bad" in mx.status_string(mx.MX_ERR_BAD_ARG)


def test_size_accounting_matches_eq1(lib):
    # Section 4.1, Eq. 1: p = e/prod(B) + m + 1 bits per element; MXInt((16,2),8,7) -> 8.25
    f = mx.fmt(32, 8)
    n = 64 * 4096
    assert 8 * (mx.mx_mant_bytes(1, 64, 4096, f) + mx.mx_exps_bytes(1, 64, 4096, f)) / n == 8.25
    # the paper's own shape: 16 columns x 2 rows per exponent, MXInt((16,2),8,7)
    f2 = mx.fmt(16, 8, block_rows=2)
    assert 8 * (mx.mx_mant_bytes(1, 64, 4096, f2) + mx.mx_exps_bytes(1, 64, 4096, f2)) / n == 8.25
    assert mx.mx_exps_bytes(1, 63, 4096, f2) == 0                     # odd number of rows
    # the fragment layout keeps that density when no padding is needed (rows % 32 == 0, cols % (4*block) == 0)
    for block, w in [(16, 4), (32, 8), (16, 6), (64, 3)]:
        f = mx.fmt(block, w)
        assert mx.mx_packed_bytes(1, 64, 1024, f) * 8 / (64 * 1024) == w + 8 / block
    # 4-bit weights with one exponent byte per 16: 0.5625 bytes per weight
    assert mx.mx_packed_bytes(1, 5120, 5120, mx.fmt(16, 4)) == 0.5625 * 5120 * 5120
    assert mx.mx_packed_bytes(3, 33, 100 * 16, mx.fmt(16, 4)) % 256 == 0
    assert mx.mx_packed_bytes(1, 32, 48, mx.fmt(32, 4)) == 0          # cols not a whole number of blocks
    assert mx.mx_mant_bytes(1, 4, 64, mx.fmt(12, 4)) == 0             # bad block


def test_matrix_layout_size_accounting(lib):
    M = mx.MX_LAYOUT_MATRIX
    # block 32/64: 6-bit codes, one per element up to 4 stored bits, two above, + one scale byte per 32 elements
    assert mx.mx_packed_bytes(1, 2048, 4096, mx.fmt(32, 8), M) == 2048 * 4096 * (12 / 8 + 1 / 32)
    assert mx.mx_packed_bytes(1, 4096, 4096, mx.fmt(32, 4), M) == 4096 * 4096 * (6 / 8 + 1 / 32)
    assert mx.mx_packed_bytes(1, 4096, 4096, mx.fmt(64, 4), M) == 4096 * 4096 * (6 / 8 + 1 / 32)
    # block 16: one bfloat16 per element + the exponent bytes, whatever the width
    for w in (2, 5, 8):
        assert mx.mx_packed_bytes(1, 2048, 2048, mx.fmt(16, w), M) == 2048 * 2048 * (2 + 1 / 16)
    # padding: rows to 32, K to 64 elements; the exponent bytes cover the logical rows only
    assert mx.mx_packed_bytes(1, 33, 48, mx.fmt(16, 4), M) == 64 * 64 * 2 + 256      # 33*3 = 99 bytes, rounded up to 256
    assert mx.mx_packed_bytes(2, 33, 48, mx.fmt(16, 4), M) == 2 * (64 * 64 * 2 + 256)
    assert mx.mx_packed_bytes(1, 32, 40, mx.fmt(16, 4), M) == 0                      # cols not a whole number of blocks
    assert mx.mx_packed_bytes(1, 32, 64, mx.fmt(8, 4), M) == 0                       # block 8 has no matrix layout


def test_bad_arguments_are_rejected_before_any_launch(lib):
    f = mx.fmt(32, 8)
    q = lambda **kw: mx.mx_quantize(kw.get("x", 256), 1, kw.get("rows", 4), kw.get("cols", 64),
                                    kw.get("rs", 64), 0, kw.get("axis", 1), kw.get("f", f),
                                    kw.get("mant", 256), kw.get("exps", 256), stream=0, check=False)
    assert q(x=0) == mx.MX_ERR_BAD_ARG                                  # null pointer
    assert q(cols=48, rs=48) == mx.MX_ERR_BAD_ARG                       # not a whole number of blocks
    assert q(rows=-1) == mx.MX_ERR_BAD_ARG
    assert q(rs=32) == mx.MX_ERR_BAD_ARG                                # row stride below cols
    assert q(axis=2) == mx.MX_ERR_BAD_ARG
    assert q(x=258) == mx.MX_ERR_BAD_ARG                                # misaligned
    assert q(f=mx.fmt(32, 9)) == mx.MX_ERR_BAD_ARG
    assert q(f=mx.fmt(32, 1)) == mx.MX_ERR_BAD_ARG
    assert q(f=mx.fmt(32, 8, exp_bits=9)) == mx.MX_ERR_BAD_ARG
    assert q(f=mx.fmt(32, 8, rounding=5)) == mx.MX_ERR_BAD_ARG
    assert q(f=mx.fmt(24, 8), cols=48, rs=48) == mx.MX_ERR_BAD_ARG
    assert q(rows=0) == mx.MX_OK                                        # empty input: nothing to do
    assert mx.mx_dequantize(0, 256, 1, 4, 64, f, 256, stream=0, check=False) == mx.MX_ERR_BAD_ARG
    assert mx.mx_pack(256, 256, 1, 4, 64, mx.fmt(8, 8), 0, 256, stream=0, check=False) == mx.MX_ERR_UNSUPPORTED
    assert mx.mx_pack(256, 256, 1, 4, 64, f, 7, 256, stream=0, check=False) == mx.MX_ERR_BAD_ARG
    assert mx.mx_pack(256, 256, 1, 4, 64, f, 0, 300, stream=0, check=False) == mx.MX_ERR_BAD_ARG  # alignment
    g = lambda **kw: mx.mx_gemm(1, kw.get("M", 16), kw.get("N", 32), kw.get("K", 64), kw.get("A", 256),
                                kw.get("fa", f), kw.get("B", 512), kw.get("fb", mx.fmt(32, 4)), 0,
                                kw.get("Y", 1024), kw.get("ldy", 32), 0, stream=0, check=False)
    assert g(fb=mx.fmt(16, 4)) == mx.MX_ERR_BAD_ARG                     # block sizes differ
    assert g(K=48) == mx.MX_ERR_BAD_ARG
    assert g(ldy=16) == mx.MX_ERR_BAD_ARG
    assert g(A=0) == mx.MX_ERR_BAD_ARG
    assert g(Y=0) == mx.MX_ERR_BAD_ARG
    assert g(fa=mx.fmt(8, 8), fb=mx.fmt(8, 4)) == mx.MX_ERR_UNSUPPORTED
    assert g(M=0) == mx.MX_OK
    assert mx.mx_linear(256, 9, 64, 64, f, 256, 512, 32, mx.fmt(32, 4), 0, 1024, 32, stream=0,
                        check=False) == mx.MX_ERR_UNSUPPORTED            # decode path is M <= 8
    # mx_linear rejects what its kernels would dereference: output, workspace and weights (all return before a launch)
    lin = lambda **kw: mx.mx_linear(kw.get("x", 256), kw.get("M", 4), 64, 64, f, kw.get("ws", 256), kw.get("B", 512), 32,
                                    mx.fmt(32, 4), 0, kw.get("Y", 1024), kw.get("ldy", 32), stream=0, check=False)
    assert lin(Y=0) == mx.MX_ERR_BAD_ARG
    assert lin(Y=1026) == mx.MX_ERR_BAD_ARG                              # not 4-byte aligned
    assert lin(B=516) == mx.MX_ERR_BAD_ARG                               # not 256-byte aligned
    assert lin(B=0) == mx.MX_ERR_BAD_ARG
    assert lin(ws=0) == mx.MX_ERR_BAD_ARG
    assert lin(ws=260) == mx.MX_ERR_BAD_ARG
    assert lin(x=0) == mx.MX_ERR_BAD_ARG
    assert lin(ldy=16) == mx.MX_ERR_BAD_ARG
    assert lin(M=0) == mx.MX_OK
    # mx_attention: output alignment, and heads that would overlap
    f16 = mx.fmt(16, 8)
    att = lambda **kw: mx.mx_attention(kw.get("batch", 2), 32, 32, 64, 256, f16, 512, f16, 768, f16, f16, 0.125,
                                       mx.MX_LAYOUT_MATRIX, kw.get("O", 1024), 64, kw.get("obs", 32 * 64), stream=0,
                                       check=False)
    assert att(O=1026) == mx.MX_ERR_BAD_ARG
    assert att(O=0) == mx.MX_ERR_BAD_ARG
    assert att(obs=31 * 64 + 63) == mx.MX_ERR_BAD_ARG                    # batch stride below (Sq-1)*ldo + D
    assert att(batch=0) == mx.MX_OK
    # mx_check_finite: its argument checks come before its launches (and before its wait)
    fin = lambda **kw: mx.mx_check_finite(kw.get("x", 256), kw.get("batch", 1), kw.get("rows", 4), 64, kw.get("rs", 64),
                                          kw.get("bs", 0), kw.get("flag", 512), stream=0)
    assert fin(x=0) == mx.MX_ERR_BAD_ARG
    assert fin(flag=0) == mx.MX_ERR_BAD_ARG
    assert fin(flag=514) == mx.MX_ERR_BAD_ARG                            # not 4-byte aligned
    assert fin(x=258) == mx.MX_ERR_BAD_ARG
    assert fin(rs=32) == mx.MX_ERR_BAD_ARG
    assert fin(batch=2, bs=100) == mx.MX_ERR_BAD_ARG                     # matrices of the batch would overlap
    assert fin(rows=0) == mx.MX_OK
    with pytest.raises(mx.MxError):
        mx.mx_quantize(0, 1, 4, 64, 64, 0, 1, f, 256, 256, stream=0)


def test_linear_workspace_bytes():
    """Workspace of mx_linear: counters + partial sums of the K slices + packed activations; 0 on bad arguments."""
    fa, fb = mx.fmt(16, 8), mx.fmt(16, 4)
    small = mx.mx_linear_workspace_bytes(1, 5120, 5120, fa, fb)
    big = mx.mx_linear_workspace_bytes(8, 5120, 13824, fa, fb)
    assert small >= 16384 + mx.mx_packed_bytes(1, 1, 5120, fa) and small % 256 == 0
    assert big > small and big < (64 << 20)
    assert mx.mx_linear_workspace_bytes(9, 5120, 5120, fa, fb) == 0
    assert mx.mx_linear_workspace_bytes(4, 5000, 5120, fa, fb) == 0      # K not a whole number of blocks
    assert mx.mx_linear_workspace_bytes(4, 5120, 5120, fa, mx.fmt(32, 4)) == 0
    assert mx.mx_linear_workspace_bytes(4, 5120, 5120, fa, fb, mx.MX_LAYOUT_MATRIX) == 0


def test_struct_layout():
    assert ctypes.sizeof(mx.mx_format) == 20
