"""Pins for the CPU oracle: everything here checks ``oracle/`` against something other than
itself -- values the paper prints, hand-worked blocks, exact rational brute force, closed forms,
invariants and library routines.  No GPU, no GPU library.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import mx_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield [c.strip() for c in line.split("|")]


# ----------------------------------------------------------------------------------------------
# Size accounting: the numbers the paper prints (Section 4.1 Eq. 1; Table 1)
# ----------------------------------------------------------------------------------------------
def test_paper_printed_sizes():
    rows = {r[0]: r for r in _rows("paper_values.txt")}
    _, B, e, m, printed, _ = rows["avg_bits_MXInt_16x2_8_7"]
    B, e, m = int(B), int(e), int(m)
    w = m + 1                                   # stored width = mantissa + sign (Eq. 1)
    x = np.zeros((3, 4 * B), np.float32)
    q, ex = orc.quantize(x, B, w, e)
    nbytes = orc.pack_bits(q, w).nbytes + ex.nbytes
    assert Fraction(8 * nbytes, x.size) == Fraction(printed)          # 8.25 bits per element
    _, B, e, m, printed, _ = rows["mem_density_MXInt8_vs_FP32"]
    bits = Fraction(int(e), int(B)) + int(m) + 1
    assert math.floor(10 * Fraction(32) / bits) / 10 == float(printed)  # 32/8.25 = 3.88 -> "3.8x"


# ----------------------------------------------------------------------------------------------
# Hand-worked blocks
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("row", list(_rows("handworked_blocks.txt")))
def test_handworked_blocks(row):
    w, rnd, xs, ebyte, qs, hexbytes = row
    w = int(w)
    x = np.array([[float(v) for v in xs.split()]], np.float32)
    q, ex = orc.quantize(x, x.shape[1], w, 8, orc.RNE if rnd == "rne" else orc.RTZ)
    assert ex.tolist() == [[int(ebyte)]]
    assert q.tolist() == [[int(v) for v in qs.split()]]
    if hexbytes != "-":
        assert orc.pack_bits(q, w).tolist() == [[int(h, 16) for h in hexbytes.split()]]


@pytest.mark.parametrize("row", list(_rows("handworked_blocks2d.txt")))
def test_handworked_two_dimensional_blocks(row):
    w, rnd, bc, br, xs, ebytes, qs = row
    x = np.array([[float(v) for v in r.split()] for r in xs.split(";")], np.float32)
    q, ex = orc.quantize(x, int(bc), int(w), 8, orc.RNE if rnd == "rne" else orc.RTZ, block_rows=int(br))
    assert ex.reshape(-1).tolist() == [int(v) for v in ebytes.split()]
    assert q.tolist() == [[int(v) for v in r.split()] for r in qs.split(";")]


def test_paper_type_16x2_size_and_structure():
    """MXInt((16,2),8,7) as the paper writes it (Section 4.1): 16 x 2 elements per exponent, 8.25 bits
    per element; every exponent covers exactly two adjacent rows and sixteen columns."""
    rows = {r[0]: r for r in _rows("paper_values.txt")}
    printed = rows["avg_bits_MXInt_16x2_8_7"][4]
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((6, 64)) * np.exp2(rng.integers(-8, 8, size=(6, 1)))).astype(np.float32)
    q, ex = orc.quantize(x, 16, 8, block_rows=2)
    assert ex.shape == (3, 4)
    assert Fraction(8 * (orc.pack_bits(q, 8).nbytes + ex.nbytes), x.size) == Fraction(printed)
    for p in range(3):
        for b in range(4):
            blk = x[2 * p:2 * p + 2, 16 * b:16 * b + 16]
            eb, qs = _brute_block(blk.reshape(-1), 8, 8, orc.RNE)
            assert ex[p, b] == eb and q[2 * p:2 * p + 2, 16 * b:16 * b + 16].reshape(-1).tolist() == qs
    # one-row blocks of 32 hold the same number of bits but are a different grouping
    q1, e1 = orc.quantize(x, 32, 8)
    assert e1.size == ex.size and not np.array_equal(orc.dequantize(q1, e1, 32, 8),
                                                     orc.dequantize(q, orc.row_exps(ex, 2), 16, 8))
    # rows that are equal pairwise: the two-row block then is the one-row block
    xx = np.repeat(x[:3], 2, axis=0)
    q2, e2 = orc.quantize(xx, 16, 5, block_rows=2)
    q3, e3 = orc.quantize(xx, 16, 5)
    assert np.array_equal(q2, q3) and np.array_equal(orc.row_exps(e2, 2), e3)


@pytest.mark.parametrize("row", list(_rows("handworked_gemm.txt")))
def test_handworked_gemm(row):
    qa, ea, wa, qb, eb, wb, val = row
    qa = np.array([[int(v) for v in qa.split()]], np.int8)
    qb = np.array([[int(v) for v in qb.split()]], np.int8)
    y = orc.gemm(qa, np.array([[int(ea)]], np.uint8), int(wa), qb, np.array([[int(eb)]], np.uint8),
                 int(wb), qa.shape[1])
    assert y[0, 0] == float(val)


@pytest.mark.parametrize("row", list(_rows("handworked_cast.txt")))
def test_handworked_cast(row):
    qs, eb, es, ws, ed, wd, rnd, qd, eb2 = row
    qs = np.array([[int(v) for v in qs.split()]], np.int8)
    q2, e2 = orc.cast(qs, np.array([[int(eb)]], np.uint8), qs.shape[1], int(ws), int(wd), int(es), int(ed), int(rnd))
    assert q2.tolist() == [[int(v) for v in qd.split()]]
    assert e2.tolist() == [[int(eb2)]]


# ----------------------------------------------------------------------------------------------
# Brute force with exact rationals: nearest representable value, ties to even, symmetric clamp
# ----------------------------------------------------------------------------------------------
def _brute_block(xs, w, e, rounding):
    """Definition only: E is the integer with 2^E <= max|x| < 2^(E+1) (found by search, clamped to the
    e-bit range); each q is the integer in [-qmax, qmax] nearest to x / 2^(E-(w-2))."""
    fx = [Fraction(float(v)) for v in xs]
    amax = max(abs(v) for v in fx)
    bias = 2 ** (e - 1) - 1
    qmax = 2 ** (w - 1) - 1
    if amax == 0:
        return 0, [0] * len(fx)
    E = -200
    while Fraction(2) ** (E + 1) <= amax:
        E += 1
    assert Fraction(2) ** E <= amax < Fraction(2) ** (E + 1)
    E = min(max(E, -bias), 2 ** e - 1 - bias)
    unit = Fraction(2) ** (E - (w - 2))
    qs = []
    for v in fx:
        t = v / unit
        if rounding == orc.RNE:
            best = None
            for cand in range(-qmax, qmax + 1):
                d = abs(t - cand)
                if best is None or d < best[0] or (d == best[0] and cand % 2 == 0 and best[1] % 2 != 0):
                    best = (d, cand)
            qs.append(best[1])
        else:
            cand = int(abs(t))                      # floor of the magnitude
            cand = min(cand, qmax)
            qs.append(cand if t >= 0 else -cand)
    return E + bias, qs


@pytest.mark.parametrize("w", [2, 3, 4, 5, 8])
@pytest.mark.parametrize("rounding", [orc.RNE, orc.RTZ])
def test_bruteforce_tiny_blocks(w, rounding):
    rng = np.random.default_rng(100 + w)
    for B in (1, 2, 3, 4):
        for trial in range(60):
            scale = 2.0 ** rng.integers(-20, 20)
            x = (rng.standard_normal(B) * scale).astype(np.float32)
            if trial % 5 == 0:                       # plant exact half-way points and a saturating max
                E = math.floor(math.log2(float(np.abs(x).max()) or 1.0))
                unit = 2.0 ** (E - (w - 2))
                x[0] = np.float32((rng.integers(0, 2 ** (w - 1)) + 0.5) * unit * rng.choice([-1, 1]))
            eb, qs = _brute_block(x, w, 8, rounding)
            q, ex = orc.quantize(x[None, :], B, w, 8, rounding)
            assert ex[0, 0] == eb and q[0].tolist() == qs, (x, w, rounding)


def test_halfway_points_dense():
    """Every half-way point (j + 1/2) units, both signs, for every width: ties go to the even code."""
    for w in range(2, 9):
        qmax = 2 ** (w - 1) - 1
        anchor = float(2 ** (w - 2)) if w > 2 else 1.0      # keeps E = w-2, i.e. unit = 1
        for j in range(0, qmax + 1):
            for sgn in (1.0, -1.0):
                x = np.array([[anchor, sgn * (j + 0.5)]], np.float32)
                if abs(x[0, 1]) >= 2 * anchor:
                    continue                                 # would move the exponent
                q, ex = orc.quantize(x, 2, w)
                assert ex[0, 0] == 127 + (w - 2)
                lo, hi = j, j + 1
                want = lo if lo % 2 == 0 else hi
                want = min(want, qmax)
                assert q[0, 1] == int(sgn) * want, (w, j, sgn)
                qz, _ = orc.quantize(x, 2, w, rounding=orc.RTZ)
                assert qz[0, 1] == int(sgn) * j


# ----------------------------------------------------------------------------------------------
# Exponent rule: closed form and invariants
# ----------------------------------------------------------------------------------------------
def test_exponent_is_floor_log2_of_block_max():
    rng = np.random.default_rng(7)
    x = (rng.standard_normal((64, 256)) * np.exp(rng.uniform(-30, 30, (64, 1)))).astype(np.float32)
    for B in (8, 16, 32):
        q, ex = orc.quantize(x, B, 6)
        amax = np.abs(x.astype(np.float64)).reshape(64, -1, B).max(-1)
        E = ex.astype(np.int64) - 127
        assert np.all(np.ldexp(1.0, E) <= amax) and np.all(amax < np.ldexp(1.0, E + 1))
        # the max-magnitude element sets the exponent: its mantissa is in the top binade
        qm = np.abs(q.astype(np.int64)).reshape(64, -1, B).max(-1)
        assert np.all(qm >= 2 ** (6 - 2)) and np.all(qm <= 2 ** 5 - 1)


def test_power_of_two_scaling_shifts_only_the_exponent():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((8, 128)).astype(np.float32)
    q0, e0 = orc.quantize(x, 16, 5)
    for j in (-40, -3, 1, 17, 60):
        q1, e1 = orc.quantize(np.ldexp(x, j).astype(np.float32), 16, 5)
        assert np.array_equal(q0, q1)
        assert np.array_equal(e0.astype(int) + j, e1.astype(int))


def test_error_bound_and_sign():
    rng = np.random.default_rng(9)
    x = rng.standard_t(3, size=(32, 512)).astype(np.float32)
    for w in (3, 4, 6, 8):
        for rounding in (orc.RNE, orc.RTZ):
            q, ex = orc.quantize(x, 32, w, rounding=rounding)
            xh = orc.dequantize(q, ex, 32, w)
            unit = np.repeat(np.ldexp(1.0, ex.astype(int) - 127 - (w - 2)), 32, axis=1)
            err = np.abs(x.astype(np.float64) - xh)
            clamped = np.abs(q) == 2 ** (w - 1) - 1
            if rounding == orc.RNE:
                assert np.all(err[~clamped] <= unit[~clamped] / 2)
            else:
                assert np.all(err[~clamped] < unit[~clamped])
                assert np.all(np.abs(xh) <= np.abs(x))          # toward zero never grows a value
            assert np.all(err[clamped] <= unit[clamped])
            assert np.all((np.sign(xh) == np.sign(x)) | (xh == 0))
            assert np.abs(q).max() <= 2 ** (w - 1) - 1            # the code -2^(w-1) is never produced


def test_roundtrip_and_idempotence():
    rng = np.random.default_rng(10)
    for w in range(2, 9):
        qmax = 2 ** (w - 1) - 1
        q = rng.integers(-qmax, qmax + 1, size=(16, 64)).astype(np.int8)
        q[:, ::16] = 2 ** (w - 2)                        # normalised: each block has a top-binade code
        ex = rng.integers(40, 200, size=(16, 4)).astype(np.uint8)
        xh = orc.dequantize(q, ex, 16, w)
        assert np.array_equal(xh, xh.astype(np.float32).astype(np.float64))   # exactly fp32 values
        q2, ex2 = orc.quantize(xh.astype(np.float32), 16, w)
        assert np.array_equal(q, q2) and np.array_equal(ex, ex2)
    x = rng.standard_normal((16, 64)).astype(np.float32)
    q, ex = orc.quantize(x, 16, 4)
    q2, ex2 = orc.quantize(orc.dequantize(q, ex, 16, 4).astype(np.float32), 16, 4)
    assert np.array_equal(q, q2) and np.array_equal(ex, ex2)


def test_widening_cast_is_value_exact():
    """Section 4 (mixed precision): a cast to a wider mantissa only extends bits."""
    rng = np.random.default_rng(11)
    x = rng.standard_normal((8, 64)).astype(np.float32)
    q4, e4 = orc.quantize(x, 16, 4)
    v = orc.dequantize(q4, e4, 16, 4).astype(np.float32)
    q7, e7 = orc.quantize(v, 16, 7)
    assert np.array_equal(e4, e7)
    assert np.array_equal(q7.astype(int), q4.astype(int) * 8)


def test_zero_subnormal_and_clamped_exponents():
    x = np.zeros((1, 16), np.float32)
    q, ex = orc.quantize(x, 16, 8)
    assert ex[0, 0] == 0 and not q.any()
    # fp32 subnormals count with their true value; E clamps at -127 (byte 0)
    tiny = np.float32(2.0 ** -140)
    x[0, 3] = tiny
    q, ex = orc.quantize(x, 16, 8)
    assert ex[0, 0] == 0                       # floor(log2) = -140 clamps to -127
    assert q[0, 3] == 0                        # 2^-140 / 2^(-127-6) = 2^-7 rounds to 0
    x[0, 3] = np.float32(2.0 ** -127)          # subnormal in fp32, exactly representable
    q, ex = orc.quantize(x, 16, 8)
    assert ex[0, 0] == 0 and q[0, 3] == 64
    # a narrow exponent (e = 4: bias 7, E in [-7, 8]) saturates large blocks and flushes small ones
    big = np.array([[1000.0, 3.0]], np.float32)
    q, ex = orc.quantize(big, 2, 4, e=4)
    assert ex[0, 0] == 15 and q.tolist() == [[7, 0]]      # unit 2^(8-2)=64: 1000/64=15.6 -> 7 ; 3/64 -> 0
    small = np.array([[2.0 ** -9, 2.0 ** -12]], np.float32)
    q, ex = orc.quantize(small, 2, 4, e=4)
    assert ex[0, 0] == 0 and q.tolist() == [[1, 0]]       # E=-7, unit 2^-9


def test_nonfinite_inputs_raise():
    x = np.ones((1, 16), np.float32)
    x[0, 5] = np.inf
    with pytest.raises(ValueError):
        orc.quantize(x, 16, 8)
    x[0, 5] = np.nan
    with pytest.raises(ValueError):
        orc.quantize(x, 16, 8)


def test_axis0_is_blocks_down_columns():
    rng = np.random.default_rng(12)
    x = rng.standard_normal((32, 5)).astype(np.float32)
    q, ex = orc.quantize(x, 16, 5, axis=0)
    assert q.shape == (5, 32) and ex.shape == (5, 2)
    for c in range(5):
        for b in range(2):
            eb, qs = _brute_block(x[16 * b:16 * b + 16, c], 5, 8, orc.RNE)
            assert ex[c, b] == eb and q[c, 16 * b:16 * b + 16].tolist() == qs


# ----------------------------------------------------------------------------------------------
# Bit packing: against numpy's own bit routines
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("w", range(2, 9))
def test_pack_bits_against_numpy_bitorder_little(w):
    rng = np.random.default_rng(20 + w)
    q = rng.integers(-(2 ** (w - 1)), 2 ** (w - 1), size=(5, 64)).astype(np.int8)
    codes = (q.astype(np.int64) & (2 ** w - 1)).astype(np.uint8)
    bits = ((codes[:, :, None] >> np.arange(w)) & 1).astype(np.uint8).reshape(5, -1)
    want = np.packbits(bits, axis=1, bitorder="little")
    got = orc.pack_bits(q, w)
    assert np.array_equal(got, want)
    assert np.array_equal(orc.unpack_bits(got, 64, w), q)


# ----------------------------------------------------------------------------------------------
# Dequantize: against 2.0**k arithmetic in exact rationals
# ----------------------------------------------------------------------------------------------
def test_dequantize_exact():
    rng = np.random.default_rng(30)
    for w in (2, 4, 8):
        q = rng.integers(-(2 ** (w - 1)) + 1, 2 ** (w - 1), size=(3, 32)).astype(np.int8)
        ex = rng.integers(0, 256, size=(3, 2)).astype(np.uint8)
        y = orc.dequantize(q, ex, 16, w)
        for r in range(3):
            for c in range(32):
                want = Fraction(int(q[r, c])) * Fraction(2) ** (int(ex[r, c // 16]) - 127 - (w - 2))
                assert Fraction(y[r, c]) == want


# ----------------------------------------------------------------------------------------------
# GEMM
# ----------------------------------------------------------------------------------------------
def _rand_mx(rng, rows, K, block, w, elo=100, ehi=140):
    qmax = 2 ** (w - 1) - 1
    q = rng.integers(-qmax, qmax + 1, size=(rows, K)).astype(np.int8)
    ex = rng.integers(elo, ehi, size=(rows, K // block)).astype(np.uint8)
    return q, ex


def test_gemm_exact_rational_tiny():
    rng = np.random.default_rng(40)
    M, N, K = 3, 4, 16
    for (wa, wb, block) in [(8, 4, 4), (3, 7, 2), (2, 2, 8)]:
        for (elo, ehi) in [(120, 132), (60, 200)]:
            qa, ea = _rand_mx(rng, M, K, block, wa, elo, ehi)
            qb, eb = _rand_mx(rng, N, K, block, wb, elo, ehi)
            y, mag = orc.gemm(qa, ea, wa, qb, eb, wb, block, want_mag=True)
            for m in range(M):
                for n in range(N):
                    tot = Fraction(0)
                    tmag = Fraction(0)
                    for b in range(K // block):
                        d = sum(int(qa[m, k]) * int(qb[n, k]) for k in range(b * block, (b + 1) * block))
                        s = int(ea[m, b]) - 127 - (wa - 2) + int(eb[n, b]) - 127 - (wb - 2)
                        tot += d * Fraction(2) ** s
                        tmag += abs(d) * Fraction(2) ** s
                    if ehi - elo < 20:
                        # few terms, narrow exponent spread: the double sums are exact
                        assert Fraction(y[m, n]) == tot
                        assert Fraction(mag[m, n]) == tmag
                    else:
                        # wide spread: each of the K/block - 1 double additions rounds once
                        assert abs(Fraction(y[m, n]) - tot) <= (K // block) * Fraction(2) ** -53 * tmag


def test_gemm_equals_float_matmul_of_dequantized_operands():
    """Section 3.2: the emulated operator is the float operator applied to the dequantized inputs."""
    rng = np.random.default_rng(41)
    M, N, K, block = 24, 40, 256, 16
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, 7] *= 50
    wt = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    for wa, wb in [(8, 4), (6, 4), (2, 8)]:
        qa, ea = orc.quantize(x, block, wa)
        qb, eb = orc.quantize(wt, block, wb)
        y, mag = orc.gemm(qa, ea, wa, qb, eb, wb, block, want_mag=True)
        ref = orc.dequantize(qa, ea, block, wa) @ orc.dequantize(qb, eb, block, wb).T   # numpy float64 matmul
        assert np.all(np.abs(y - ref) <= 1e-13 * mag)
        assert np.all(mag >= np.abs(y) * (1 - 1e-12))


def test_gemm_special_cases():
    rng = np.random.default_rng(42)
    M, K, block, wa = 6, 64, 16, 7
    qa, ea = _rand_mx(rng, M, K, block, wa)
    # identity weights: value 1.0 = code 2^(w-2) with E = 0  ->  output equals the dequantized activations
    wb = 4
    qb = (np.eye(K, dtype=np.int8) * 2 ** (wb - 2)).astype(np.int8)
    eb = np.full((K, K // block), 127, np.uint8)
    y = orc.gemm(qa, ea, wa, qb, eb, wb, block)
    assert np.array_equal(y, orc.dequantize(qa, ea, block, wa))
    # all exponents equal: one integer matrix product times one power of two
    qb, _ = _rand_mx(rng, 5, K, block, wb)
    ea2 = np.full_like(ea, 130)
    eb2 = np.full((5, K // block), 120, np.uint8)
    y = orc.gemm(qa, ea2, wa, qb, eb2, wb, block)
    want = (qa.astype(np.int64) @ qb.astype(np.int64).T) * 2.0 ** ((130 - 127 - 5) + (120 - 127 - 2))
    assert np.array_equal(y, want)
    # one block per row (block = K): per-row times per-column scaling of the integer product
    ea3 = rng.integers(110, 140, size=(M, 1)).astype(np.uint8)
    eb3 = rng.integers(110, 140, size=(5, 1)).astype(np.uint8)
    y = orc.gemm(qa, ea3, wa, qb, eb3, wb, K)
    want = (qa.astype(np.int64) @ qb.astype(np.int64).T) * np.ldexp(1.0, ea3.astype(int) - 132) \
        * np.ldexp(1.0, eb3.astype(int).T - 129)
    assert np.array_equal(y, want)
    # transposing the roles of the operands transposes the result
    y_t = orc.gemm(qb, eb3, wb, qa, ea3, wa, K)
    assert np.array_equal(y_t, y.T)


def test_gemm_row_window():
    rng = np.random.default_rng(43)
    qa, ea = _rand_mx(rng, 10, 32, 16, 8)
    qb, eb = _rand_mx(rng, 7, 32, 16, 4)
    full = orc.gemm(qa, ea, 8, qb, eb, 4, 16)
    part = orc.gemm(qa, ea, 8, qb, eb, 4, 16, rows=(3, 6))
    assert np.array_equal(part[3:6], full[3:6]) and np.isnan(part[:3]).all() and np.isnan(part[6:]).all()


def test_linear_matches_float_linear_within_quantization_error():
    """Sanity of the whole chain on config-1-shaped data: the MXInt linear tracks the fp64 linear to
    the accuracy the formats allow (8-bit activations, 4-bit weights)."""
    from paper_2307_15517_amd import inputs
    case = inputs.single_linear()[0]
    x, wt = inputs.make(case)
    y = orc.linear(x, wt, case.block, case.wx, case.ww)
    ref = x.astype(np.float64) @ wt.astype(np.float64).T
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    assert 0.01 < rel < 0.2            # 4-bit weights: ~10 % error; not zero, not garbage


# ----------------------------------------------------------------------------------------------
# Width cast: it must equal quantizing the exact values (two independent routes: integer shifts
# there, exact rationals / the float quantizer here)
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("ws", [2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("wd", [2, 3, 4, 5, 6, 7, 8])
def test_cast_equals_quantizing_the_exact_values(ws, wd):
    rng = np.random.default_rng(1000 + 10 * ws + wd)
    block = 16
    q = rng.integers(-(2 ** (ws - 1)), 2 ** (ws - 1), size=(40, 4 * block)).astype(np.int8)
    q[::3] //= 4                                        # blocks that are not normalised
    q[5] = 0                                            # zero blocks
    ex = rng.integers(20, 230, size=(40, 4)).astype(np.uint8)        # exact in fp32
    x = orc.dequantize(q, ex, block, ws)
    x32 = x.astype(np.float32)
    assert np.array_equal(x32.astype(np.float64), x)
    for rounding in (orc.RNE, orc.RTZ):
        want_q, want_e = orc.quantize(x32, block, wd, 8, rounding)
        got_q, got_e = orc.cast(q, ex, block, ws, wd, 8, 8, rounding)
        assert np.array_equal(got_q, want_q) and np.array_equal(got_e, want_e)


def test_cast_brute_force_small_blocks():
    """Exact rationals on every 2-element block of 4-bit mantissas, to 3 and to 6 bits, both roundings."""
    for wd in (3, 6):
        for rounding in (orc.RNE, orc.RTZ):
            for a in range(-8, 8):
                for b in range(-8, 8):
                    q = np.array([[a, b]], np.int8)
                    ex = np.array([[130]], np.uint8)
                    vals = [Fraction(a) * Fraction(2) ** (3 - 2), Fraction(b) * Fraction(2) ** (3 - 2)]   # E = 3, ws = 4
                    eb, qs = _brute_block([float(v) for v in vals], wd, 8, rounding)
                    got_q, got_e = orc.cast(q, ex, 2, 4, wd, 8, 8, rounding)
                    assert got_q.tolist() == [qs] and got_e.tolist() == [[eb]], (a, b, wd, rounding)


def test_cast_invariants():
    rng = np.random.default_rng(77)
    block = 32
    x = (rng.standard_normal((30, 4 * block)) * np.exp2(rng.integers(-20, 20, size=(30, 1)))).astype(np.float32)
    for w in range(2, 9):
        q, ex = orc.quantize(x, block, w)
        same_q, same_e = orc.cast(q, ex, block, w, w)
        assert np.array_equal(same_q, q) and np.array_equal(same_e, ex)          # identity on quantizer output
        for wide in range(w, 9):
            uq, ue = orc.cast(q, ex, block, w, wide)                              # widening is exact ...
            assert np.array_equal(orc.dequantize(uq, ue, block, wide), orc.dequantize(q, ex, block, w))
            bq, be = orc.cast(uq, ue, block, wide, w)                             # ... and narrowing back undoes it
            assert np.array_equal(bq, q) and np.array_equal(be, ex)
    # narrowing error: at most half a destination unit (nearest), less than one (truncation)
    q8, e8 = orc.quantize(x, block, 8)
    for wd in range(2, 8):
        for rounding, lim in ((orc.RNE, 0.5), (orc.RTZ, 1.0)):
            nq, ne = orc.cast(q8, e8, block, 8, wd, 8, 8, rounding)
            unit = np.repeat(np.ldexp(1.0, ne.astype(int) - 127 - (wd - 2)), block, axis=1)
            err = np.abs(orc.dequantize(nq, ne, block, wd) - orc.dequantize(q8, e8, block, 8))
            sat = np.abs(nq) == 2 ** (wd - 1) - 1
            assert np.all(err[~sat] <= lim * unit[~sat]) and np.all(err[sat] <= unit[sat])


# ----------------------------------------------------------------------------------------------
# The emulated linear layer with bias and output quantizer (Section 3.2; the LinearOp of Fig. 2b)
# ----------------------------------------------------------------------------------------------
def test_linear_q_hand_worked_and_composition():
    # x = [1, 0.5 | 0.25, 0.25], W row 0 = [1, 1 | 2, -2], row 1 = [0.5, 0 | 0, 1]; blocks of 2; 8-bit everything:
    # every value is exact in its block, so y = [1.5 + 0, 0.5 + 0.25] = [1.5, 0.75]; bias [0.25, -0.75] -> [1.75, 0.0]
    x = np.array([[1.0, 0.5, 0.25, 0.25]], np.float32)
    wt = np.array([[1.0, 1.0, 2.0, -2.0], [0.5, 0.0, 0.0, 1.0]], np.float32)
    bias = np.array([0.25, -0.75], np.float32)
    qo, eo, y, mag = orc.linear_q(x, wt, bias, 2, 8, 8, 8, 4)
    assert y.tolist() == [[1.75, 0.0]]
    # output block [1.75, 0]: E = 0 (byte 127), 4 bits: unit 0.25 -> q = [7, 0]
    assert qo.tolist() == [[7, 0]] and eo.tolist() == [[127]]
    assert mag.tolist() == [[1.5 + 0.0 + 0.25, 0.5 + 0.25 + 0.75]]      # |block sums| + |bias|
    # composition: the same as the separately pinned pieces
    rng = np.random.default_rng(11)
    x = rng.standard_normal((6, 64)).astype(np.float32)
    wt = (rng.standard_normal((32, 64)) * 0.1).astype(np.float32)
    b = rng.standard_normal(32).astype(np.float32)
    for br in (1, 2):
        qo, eo, y, _ = orc.linear_q(x, wt, b, 16, 8, 4, 4, 6, block_rows=br)
        qa, ea = orc.quantize(x, 16, 8, block_rows=br)
        qb, eb = orc.quantize(wt, 16, 4, block_rows=br)
        ref = orc.dequantize(qa, orc.row_exps(ea, br), 16, 8) @ orc.dequantize(qb, orc.row_exps(eb, br), 16, 4).T
        bq, be = orc.quantize(b.reshape(1, -1), 16, 4)
        ref = ref + orc.dequantize(bq, be, 16, 4)
        assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)
        q2, e2 = orc.quantize(y.astype(np.float32), 16, 6, block_rows=br)
        assert np.array_equal(qo, q2) and np.array_equal(eo, e2)


def test_cast_two_row_blocks_equals_quantizing_the_exact_values():
    rng = np.random.default_rng(2024)
    block, R = 16, 2
    for ws, wd in [(8, 4), (4, 8), (6, 3), (5, 5)]:
        q = rng.integers(-(2 ** (ws - 1)), 2 ** (ws - 1), size=(12, 4 * block)).astype(np.int8)
        q[::4] //= 4
        ex = rng.integers(40, 200, size=(6, 4)).astype(np.uint8)
        x = orc.dequantize(q, orc.row_exps(ex, R), block, ws).astype(np.float32)
        for rounding in (orc.RNE, orc.RTZ):
            want_q, want_e = orc.quantize(x, block, wd, 8, rounding, block_rows=R)
            got_q, got_e = orc.cast(q, ex, block, ws, wd, 8, 8, rounding, block_rows=R)
            assert np.array_equal(got_q, want_q) and np.array_equal(got_e, want_e)


# ----------------------------------------------------------------------------------------------
# Attention with both products in MXInt (Fig. 1; Section 3.2): closed forms and hand-worked rows
# ----------------------------------------------------------------------------------------------
def _vdeq(V, block, wv):
    vq, ve = orc.quantize(V, block, wv, axis=0)               # quantization of V^T
    return orc.dequantize(vq, ve, block, wv).T                # [Sk, D]


def test_attention_uniform_scores_average_the_values():
    """All scores equal -> every probability is 1/Sk; with Sk a power of two that is an MXInt value, so the
    output is exactly the mean over the keys of the quantized V."""
    rng = np.random.default_rng(5)
    Sk, D = 32, 48
    Q = np.zeros((5, D), np.float32)
    K = rng.standard_normal((Sk, D)).astype(np.float32)
    V = rng.standard_normal((Sk, D)).astype(np.float32)
    for wp in (2, 5, 8):
        O, info = orc.attention(Q, K, V, 16, 8, 8, wp, 6, scale=0.3)
        assert np.all(info["P"] == 1.0 / Sk)
        want = _vdeq(V, 16, 6).sum(axis=0) / Sk               # dyadic numbers: exact in float64
        assert np.array_equal(O, np.broadcast_to(want, O.shape))


def test_attention_dominant_key_selects_its_value_row():
    """Query i matches key perm(i) by a margin of 2000: softmax is exactly one-hot in float64, the quantized
    probability is exactly 1, and row i of the output is row perm(i) of the quantized V.  A softmax along the
    wrong axis, a transposed operand or a swapped index would pick other rows."""
    rng = np.random.default_rng(6)
    n = 32
    perm = rng.permutation(n)
    K = np.eye(n, dtype=np.float32)
    Q = np.zeros((n, n), np.float32)
    Q[np.arange(n), perm] = 2000.0                            # 125 * 2^4: exact at width 8
    V = rng.standard_normal((n, 16)).astype(np.float32)
    O, info = orc.attention(Q, K, V, 16, 8, 8, 4, 8, scale=1.0)
    onehot = np.zeros((n, n))
    onehot[np.arange(n), perm] = 1.0
    assert np.array_equal(info["P"], onehot)
    assert np.array_equal(O, _vdeq(V, 16, 8)[perm])


def test_attention_hand_worked_three_quarters():
    """Scores (2, 1, -1024 x 14) with scale ln 3: probabilities (3/4, 1/4, 0, ...).
    Width 4: E = -1, mantissas 6 and 2 (0.75 and 0.25 exactly)  -> O = 0.75 v0 + 0.25 v1.
    Width 2: 0.75 * 2 = 1.5 rounds to 2 and is clamped to 1; 0.25 * 2 = 0.5 is a tie and goes to the even
    mantissa 0                                                  -> O = 0.5 v0."""
    Sk, D = 16, 16
    K = np.zeros((Sk, D), np.float32)
    K[:, 0] = -1024.0
    K[0, 0], K[1, 0] = 2.0, 1.0
    Q = np.zeros((3, D), np.float32)
    Q[:, 0] = 1.0
    V = np.zeros((Sk, D), np.float32)
    V[0, :4] = [1.0, -2.0, 0.5, 4.0]
    V[1, :4] = [3.0, 1.0, -0.5, -4.0]
    V[2:, :] = 7.0                                            # must not leak in: its probability is 0
    O, info = orc.attention(Q, K, V, 16, 8, 8, 4, 8, scale=math.log(3.0))
    assert np.allclose(info["P"][:, :2], [[0.75, 0.25]] * 3, rtol=0, atol=1e-15)
    assert info["pq"][0, :3].tolist() == [6, 2, 0] and info["pe"][0, 0] == 127 - 1
    assert np.array_equal(O[:, :4], [[1.5, -1.25, 0.25, 2.0]] * 3)
    assert np.all(O[:, 4:] == 0.0)
    O2, info2 = orc.attention(Q, K, V, 16, 8, 8, 2, 8, scale=math.log(3.0))
    assert info2["pq"][0, :3].tolist() == [1, 0, 0]
    assert np.array_equal(O2[:, :4], [[0.5, -1.0, 0.25, 2.0]] * 3)


def test_attention_steps_against_library_routines():
    """Step by step against routines that are not the oracle's own: scores against the float matmul of the
    dequantized operands, softmax against scipy's, the second product against the float matmul of the
    dequantized probabilities and values; and the row window returns the same rows."""
    from scipy.special import softmax
    rng = np.random.default_rng(7)
    Sq, Sk, D = 24, 80, 64
    Q = rng.standard_normal((Sq, D)).astype(np.float32)
    K = rng.standard_normal((Sk, D)).astype(np.float32)
    V = rng.standard_normal((Sk, D)).astype(np.float32)
    Q[:, 3] *= 50.0
    O, info = orc.attention(Q, K, V, 16, 7, 6, 5, 3, scale=D ** -0.5)
    qq, qe = orc.quantize(Q, 16, 7)
    kq, ke = orc.quantize(K, 16, 6)
    S = orc.dequantize(qq, qe, 16, 7) @ orc.dequantize(kq, ke, 16, 6).T
    assert np.allclose(info["S"], S, rtol=1e-12, atol=1e-12)
    P = softmax(S * D ** -0.5, axis=1)
    assert np.allclose(info["P"], P, rtol=1e-12, atol=1e-300)
    assert np.allclose(info["P"].sum(axis=1), 1.0, rtol=1e-13)
    pd = orc.dequantize(info["pq"], info["pe"], 16, 5)
    assert np.all(np.abs(pd - P) <= 2.0 ** (np.floor(np.log2(P.reshape(Sq, -1, 16).max(axis=2))) - 3).repeat(16, axis=1))
    assert np.allclose(O, pd @ _vdeq(V, 16, 3), rtol=1e-12, atol=1e-12)
    O2, _ = orc.attention(Q, K, V, 16, 7, 6, 5, 3, scale=D ** -0.5, rows=(8, 16))
    assert np.array_equal(O2[8:16], O[8:16]) and np.all(np.isnan(O2[:8])) and np.all(np.isnan(O2[16:]))


def test_attention_narrow_exponent_for_p_and_v():
    """A separate exponent width for P and V (e_pv).  Hand-worked: with e_pv = 4 the smallest block exponent
    is -7, so a block of probabilities whose maximum is 2^-12 is held with exponent -7 -- at width 8 its
    mantissas are p * 2^13 = 2, exact -- and a block whose maximum is 2^-20 loses everything but does not
    wrap.  V saturates the other way: 1000 needs exponent 9 and e_pv = 4 stops at 8, so the mantissa clamps
    at 127 * 2^(8-6) = 508.  Then each step against routines that are not the oracle's: the second product is
    the float matmul of the operands quantized with e_pv, and e_pv = e reproduces the default call."""
    from scipy.special import softmax
    Sk, D = 32, 16
    K = np.zeros((Sk, D), np.float32)
    K[:, 0] = [0.0] + [-12.0] * 15 + [-20.0] * 16          # log2 of the unnormalised probabilities
    Q = np.zeros((2, D), np.float32)
    Q[:, 0] = 1.0
    V = np.zeros((Sk, D), np.float32)
    V[0, 0], V[1, 0], V[16, 0] = 1000.0, 1.0, 1.0
    O, info = orc.attention(Q, K, V, 16, 8, 8, 8, 8, scale=math.log(2.0), e_pv=4)
    Z = 1.0 + 15 * 2.0 ** -12 + 16 * 2.0 ** -20
    assert np.allclose(info["P"][0, :2], [1 / Z, 2.0 ** -12 / Z], rtol=1e-14)
    assert info["pe"][0].tolist() == [7 - 1, 0]                          # E = -1 (p0 just below 1); clamped at -7
    assert info["pq"][0, 16:].tolist() == [0] * 16                      # 2^-20 * 2^13 rounds to 0
    assert info["ve"][0].tolist() == [15, 7]                             # E = 8 (clamped from 9); E = 0
    assert info["vq"][0, 0] == 127 and info["vq"][0, 1] == 0 and info["vq"][0, 16] == 64
    p0 = float(info["pq"][0, 0]) * 2.0 ** (-1 - 6)
    p1 = float(info["pq"][0, 1]) * 2.0 ** (-1 - 6)
    assert info["pq"][0, 1] == 0                                         # 2^-12 shares the block of p0: below half a step
    assert O[0, 0] == p0 * 508.0 + p1 * 0.0
    rng = np.random.default_rng(11)
    Sq, Sk, D = 16, 64, 32
    Q = rng.standard_normal((Sq, D)).astype(np.float32)
    K = rng.standard_normal((Sk, D)).astype(np.float32)
    V = (rng.standard_normal((Sk, D)) * 300.0).astype(np.float32)
    O, info = orc.attention(Q, K, V, 16, 7, 6, 5, 4, scale=1.0, e_pv=4)
    P = softmax(info["S"], axis=1)
    pq, pe = orc.quantize(P.astype(np.float32), 16, 5, 4)
    vq, ve = orc.quantize(V, 16, 4, 4, axis=0)
    assert np.array_equal(pq, info["pq"]) and np.array_equal(pe, info["pe"])
    assert np.array_equal(vq, info["vq"]) and np.array_equal(ve, info["ve"])
    assert pe.min() == 0 and ve.max() == 15                              # both clamps are reached here
    assert np.allclose(O, orc.dequantize(pq, pe, 16, 5, 4) @ orc.dequantize(vq, ve, 16, 4, 4).T, rtol=1e-12, atol=1e-12)
    Oa, _ = orc.attention(Q, K, V, 16, 7, 6, 5, 4, scale=1.0, e_pv=8)
    Ob, _ = orc.attention(Q, K, V, 16, 7, 6, 5, 4, scale=1.0)
    assert np.array_equal(Oa, Ob) and not np.array_equal(Oa, O)


def test_attention_two_row_blocks_pairs_of_equal_rows_change_nothing():
    """The paper's block shape (block, 2) (Section 3, the MASE IR example; Section 4.1) in the attention layer.  When rows 2i and 2i+1 of
    every quantized matrix are equal (queries, keys, and the columns of V, which are the rows of V^T), a
    two-row block holds the same values twice, so its maximum, exponent and mantissas are those of the
    one-row blocks: the outputs are identical."""
    rng = np.random.default_rng(11)
    Sq, Sk, D = 12, 32, 32
    Q = np.repeat(rng.standard_normal((Sq // 2, D)), 2, axis=0).astype(np.float32)
    K = np.repeat(rng.standard_normal((Sk // 2, D)) * np.exp2(rng.integers(-3, 4, (Sk // 2, 1))), 2, axis=0).astype(np.float32)
    V = np.repeat(rng.standard_normal((Sk, D // 2)) * np.exp2(rng.integers(-3, 4, (1, D // 2))), 2, axis=1).astype(np.float32)
    O1, i1 = orc.attention(Q, K, V, 16, 7, 6, 5, 4, scale=0.4)
    O2, i2 = orc.attention(Q, K, V, 16, 7, 6, 5, 4, scale=0.4, block_rows=2)
    assert np.array_equal(O1, O2) and np.array_equal(i1["pq"], i2["pq"]) and np.array_equal(i1["pe"], i2["pe"])
    assert np.array_equal(i1["vq"], i2["vq"]) and np.array_equal(i1["ve"], i2["ve"])
    # ordinary inputs: the exponent of the pair (2i, 2i+1) is the larger of the two rows' own exponents
    # (floor(log2) of the larger maximum), for the probabilities and for V^T
    Q, K, V = (rng.standard_normal(x.shape).astype(np.float32) for x in (Q, K, V))
    _, j1 = orc.attention(Q, K, V, 16, 7, 6, 5, 4, scale=0.4)
    _, j2 = orc.attention(Q, K, V, 16, 7, 6, 5, 4, scale=0.4, block_rows=2)
    for key in ("pe", "ve"):
        pair_max = np.maximum(j1[key][0::2], j1[key][1::2])
        assert np.array_equal(j2[key][0::2], pair_max) and np.array_equal(j2[key][1::2], pair_max)
        assert not np.array_equal(j1[key], j2[key])


def test_attention_two_row_blocks_hand_worked():
    """Query 0 matches key 0 by a wide margin (P = 1, 0, 0, ...), query 1 is zero (P = 1/16 each), ternary
    probabilities (width 2: one step = 2^E).  One-row blocks: row 1 has E = -4, mantissa 1 everywhere, and its
    output is the mean of the quantized V.  Two-row blocks: rows 0 and 1 share E = 0 from the 1 in row 0, so
    row 1's 1/16 is far below half a step and quantizes to 0: its output is exactly 0, row 0 is unchanged."""
    Sk, D = 16, 16
    rng = np.random.default_rng(12)
    K = np.zeros((Sk, D), np.float32)
    K[0, 0] = 1.0
    Q = np.zeros((2, D), np.float32)
    Q[0, 0] = 2000.0
    V = rng.standard_normal((Sk, D)).astype(np.float32)
    vd = _vdeq(V, 16, 8)
    O1, i1 = orc.attention(Q, K, V, 16, 8, 8, 2, 8, scale=1.0)
    assert i1["pq"][1].tolist() == [1] * 16 and i1["pe"][1, 0] == 127 - 4
    assert np.array_equal(O1[0], vd[0]) and np.array_equal(O1[1], vd.sum(axis=0) / 16)
    O2, i2 = orc.attention(Q, K, V, 16, 8, 8, 2, 8, scale=1.0, block_rows=2)
    assert i2["pe"][:, 0].tolist() == [127, 127] and i2["pq"][1].tolist() == [0] * 16
    # V^T in two-row blocks: columns 2j and 2j+1 of V share exponents, row 0 of the output is that V row 0
    vq, ve = orc.quantize(np.ascontiguousarray(V.T), 16, 8, block_rows=2)
    vd2 = orc.dequantize(vq, orc.row_exps(ve, 2), 16, 8).T
    assert np.array_equal(O2[0], vd2[0]) and np.all(O2[1] == 0.0)


# ----------------------------------------------------------------------------------------------
# Block Minifloat and Block Logarithm (Section 2): the format's value set written out, brute force
# ----------------------------------------------------------------------------------------------
def _minifloat_values(T, e, m):
    """Every non-negative representable value of a block with top exponent T, as exact fractions, indexed
    by its code integer (c << m | f): the definition, enumerated."""
    cmax = 2 ** e - 1
    vals = []
    for c in range(cmax + 1):
        for f in range(2 ** m):
            if c >= 1:
                vals.append(Fraction(2) ** (c - cmax + T) * (1 + Fraction(f, 2 ** m)))
            else:
                vals.append(Fraction(2) ** (1 - cmax + T) * Fraction(f, 2 ** m))
    return vals


def _minifloat_nearest(x, vals, rounding):
    """Code of the representable value nearest to |x| (ties: even code; RTZ: largest value <= |x|)."""
    a = abs(Fraction(float(x)))
    if rounding == orc.RTZ:
        return max(i for i, v in enumerate(vals) if v <= a)
    best = min(range(len(vals)), key=lambda i: (abs(vals[i] - a), i & 1))
    return best


@pytest.mark.parametrize("e,m", [(2, 1), (3, 0), (2, 0), (3, 2), (4, 3), (1, 2)])
def test_minifloat_brute_force(e, m):
    """Against the enumerated value set: the shared top exponent is the smallest one whose value set reaches
    the rounded block maximum, and every element takes the nearest value (ties to the even code)."""
    rng = np.random.default_rng(100 * e + m)
    block = 8
    x = (rng.standard_normal((40, 2 * block)) * np.exp2(rng.integers(-6, 6, size=(40, 1)))).astype(np.float32)
    x[0, :block] = 0.0
    x[1, 3] = 0.0
    # exact ties and exact representable values, in a block whose maximum pins T = 0
    vals0 = _minifloat_values(0, e, m)
    mids = [float((vals0[i] + vals0[i + 1]) / 2) for i in range(len(vals0) - 1)]
    x[2, :block] = (mids + [1.0] * block)[:block]
    x[2, block - 1] = 1.0
    x[3, :block] = ([float(v) for v in vals0[-block + 1:]] + [1.0] * block)[:block]
    for rounding in (orc.RNE, orc.RTZ):
        codes, shared = orc.quantize_minifloat(x, block, e, m, rounding)
        for r in range(x.shape[0]):
            for b in range(2):
                blk = x[r, b * block:(b + 1) * block]
                amax = np.abs(blk).max()
                if amax == 0:
                    assert shared[r, b] == 0 and not codes[r, b * block:(b + 1) * block].any()
                    continue
                T = int(shared[r, b]) - 127
                vals = _minifloat_values(T, e, m)
                a = Fraction(float(amax))
                # T is minimal: with T - 1 the maximum would have to saturate (or, for RTZ, lie above the range)
                if rounding == orc.RNE:
                    top = vals[-1]
                    nxt = Fraction(2) ** (T + 1)
                    assert a < (top + nxt) / 2
                    lower = _minifloat_values(T - 1, e, m)
                    assert a >= (lower[-1] + Fraction(2) ** T) / 2
                else:
                    assert Fraction(2) ** T <= a < Fraction(2) ** (T + 1)
                for i, xv in enumerate(blk):
                    code = int(codes[r, b * block + i])
                    sign, mag = code >> (e + m), code & (2 ** (e + m) - 1)
                    assert sign == int(np.signbit(xv))
                    assert mag == _minifloat_nearest(xv, vals, rounding), (r, b, i, float(xv), T)


def test_minifloat_hand_worked_blocks():
    """BMF(e=2, m=1), block of 4, maximum 3.0: T = 1, cmax = 3, values 0, .25 | .5, .75 | 1, 1.5 | 2, 3.
    3.0 -> c=3 f=1 (code 7); 1.25 is a tie between 1 (code 4) and 1.5 (code 5) -> 1; -0.6 -> -0.5 (sign, code 2);
    0.1 -> nearer 0 than 0.25 -> 0.
    BL(e=2): maximum 3.0 is at the midpoint of 2 and 4 -> T = 2 (values 0, 1, 2, 4), 3.0 is a tie between 2 (code 2)
    and 4 (code 3) -> 2; 1.5 a tie between 1 (code 1) and 2 (code 2) -> 2; 0.5 a tie between 0 (code 0) and 1 -> 0."""
    x = np.array([[3.0, 1.25, -0.6, 0.1]], np.float32)
    codes, shared = orc.quantize_minifloat(x, 4, 2, 1)
    assert shared.tolist() == [[128]] and codes.tolist() == [[7, 4, 8 + 2, 0]]
    assert orc.dequantize_minifloat(codes, shared, 4, 2, 1).tolist() == [[3.0, 1.0, -0.5, 0.0]]
    x = np.array([[3.0, 1.5, -0.5, 0.7]], np.float32)
    codes, shared = orc.quantize_minifloat(x, 4, 2, 0)
    assert shared.tolist() == [[129]] and codes.tolist() == [[2, 2, 0 + 4, 1]]
    assert orc.dequantize_minifloat(codes, shared, 4, 2, 0).tolist() == [[2.0, 2.0, -0.0, 1.0]]
    codes, shared = orc.quantize_minifloat(x, 4, 2, 0, orc.RTZ)                # toward zero: T = 1, values 0, .5, 1, 2
    assert shared.tolist() == [[128]] and codes.tolist() == [[3, 2, 4 + 1, 1]]


def test_minifloat_invariants():
    rng = np.random.default_rng(9)
    for e, m, block in [(4, 3, 16), (3, 4, 32), (7, 0, 16), (5, 2, 8)]:
        x = (rng.standard_normal((32, 4 * block)) * np.exp2(rng.integers(-20, 20, size=(32, 1)))).astype(np.float32)
        codes, shared = orc.quantize_minifloat(x, block, e, m)
        y = orc.dequantize_minifloat(codes, shared, block, e, m)
        # representable values come back exactly, and quantizing them again changes nothing
        c2, s2 = orc.quantize_minifloat(y.astype(np.float32), block, e, m)
        assert np.array_equal(c2, codes) and np.array_equal(s2, shared)
        # error at most half a step of the value's binade (steps are 2^(k-m), k >= the smallest binade)
        T = shared.astype(int).repeat(block, axis=1) - 127
        k = np.maximum(np.floor(np.log2(np.maximum(np.abs(x.astype(np.float64)), 1e-300))), T - (2 ** e - 1) + 1)
        assert np.all(np.abs(y - x) <= np.exp2(k - m - 1) * (1 + 1e-12))
        assert np.array_equal(np.signbit(y), np.signbit(x))
        # scaling by a power of two moves only the shared byte
        c3, s3 = orc.quantize_minifloat(x * 8.0, block, e, m)
        assert np.array_equal(c3, codes) and np.array_equal(s3.astype(int), shared.astype(int) + 3)
        # the block maximum lands in the top binade or one below its top (when T was raised for the carry)
        cfield = (codes >> m) & (2 ** e - 1)
        assert np.all(cfield.reshape(32, 4, block).max(axis=2) >= 2 ** e - 2)
        if m == 0:                                       # block logarithm: powers of two or zero
            nz = y != 0
            assert np.all(np.exp2(np.round(np.log2(np.abs(y[nz])))) == np.abs(y[nz]))
    with pytest.raises(Exception):
        orc.quantize_minifloat(np.array([[np.inf, 0, 0, 0]], np.float32), 4, 3, 2)
