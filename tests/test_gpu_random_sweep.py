"""Randomly drawn shapes and formats through the helpers of test_gpu_parity: the same oracle comparisons, on
cases nobody picked by hand.  Every case is printed before it runs (pytest -s shows it)."""
import numpy as np
import pytest
import torch

import test_gpu_parity as T

pytestmark = pytest.mark.gpu
mx, orc, say = T.mx, T.orc, T.say
SEEDS = [1, 2, 3]


@pytest.mark.parametrize("seed", SEEDS)
def test_random_quantizer(seed):
    """Both axes, one- and two-row blocks, all block sizes, widths, exponent widths and rounding modes, ragged shapes,
    zeros sprinkled in: bit-exact."""
    rng = np.random.default_rng(1000 * seed + 0)
    for it in range(120):
        block = int(rng.choice([8, 16, 32, 64])); w = int(rng.integers(2, 9)); e = int(rng.choice([8, 8, 8, 5, 3]))
        rounding = int(rng.integers(0, 2)); axis = int(rng.integers(0, 2)); R = int(rng.choice([1, 1, 2]))
        nb = int(rng.integers(1, 40))
        if axis == 1:
            rows, cols = int(rng.integers(1, 300)), nb * block
            if R == 2: rows += rows % 2
        else:
            rows, cols = nb * block, int(rng.integers(1, 200))
            if R == 2: cols += cols % 2
        say("quantize", it, dict(block=block, w=w, e=e, rounding=rounding, axis=axis, R=R, rows=rows, cols=cols))
        x = (rng.standard_normal((rows, cols)) * np.exp2(rng.integers(-20, 20, size=(rows, 1)))).astype(np.float32)
        x[rng.random((rows, cols)) < 0.05] = 0.0
        f = mx.fmt(block, w, e, rounding, R)
        mant, exps = mx.quantize(T.dev(x), f, axis=axis)
        torch.cuda.synchronize()
        xo = x if axis == 1 else np.ascontiguousarray(x.T)
        q, ex = orc.quantize(xo, block, w, e, rounding, block_rows=R)
        assert np.array_equal(T.host(exps), ex.reshape(-1)) and np.array_equal(T.host(mant), orc.pack_bits(q, w).reshape(-1))


@pytest.mark.parametrize("seed", SEEDS)
def test_random_products(seed):
    """Both layouts, all block sizes and width pairs, decode and tiled row counts, ragged N and K, batches."""
    rng = np.random.default_rng(1000 * seed + 1)
    for it in range(60):
        layout = int(rng.integers(0, 2)); block = int(rng.choice([16, 32, 64])); wa = int(rng.integers(2, 9)); wb = int(rng.integers(2, 9))
        M = int(rng.choice([1, 2, 3, 5, 8, 9, 31, 33, 100, 129, 257])); N = int(rng.integers(1, 600)); K = int(rng.integers(1, 30)) * block
        batch = int(rng.choice([1, 1, 2]))
        say("gemm", it, dict(layout=layout, block=block, wa=wa, wb=wb, M=M, N=N, K=K, batch=batch))
        ops_a = [T.random_operand(rng, M, K, block, wa, 118, 130) for _ in range(batch)]
        ops_b = [T.random_operand(rng, N, K, block, wb, 110, 125) for _ in range(batch)]
        qa = np.stack([o[0] for o in ops_a]); ea = np.stack([o[1] for o in ops_a])
        qb = np.stack([o[0] for o in ops_b]); eb = np.stack([o[1] for o in ops_b])
        A, fa = T.gpu_operand(qa, ea, block, wa, batch, layout)
        B, fb = T.gpu_operand(qb, eb, block, wb, batch, layout)
        y = mx.gemm(A, fa, B, fb, M, N, K, batch=batch, layout=layout)
        torch.cuda.synchronize()
        for b in range(batch):
            y_ref, mag = orc.gemm(qa[b], ea[b], wa, qb[b], eb[b], wb, block, want_mag=True)
            me = T.product_magnitude(qa[b], ea[b], wa, qb[b], eb[b], wb, block) if layout == 1 else None
            T.check_product(T.host(y)[b], y_ref, mag, "random product", me)


@pytest.mark.parametrize("seed", SEEDS)
def test_random_decode_linear(seed):
    """mx_linear over row counts 1..8, formats, ragged K and N, aligned and unaligned rows."""
    rng = np.random.default_rng(1000 * seed + 2)
    for it in range(30):
        block = int(rng.choice([16, 32, 64])); wx = int(rng.integers(2, 9)); ww = int(rng.integers(2, 9)); M = int(rng.integers(1, 9))
        K = int(rng.integers(1, 60)) * block; N = int(rng.integers(1, 300)); off = int(rng.integers(0, 2))
        say("linear", it, dict(block=block, wx=wx, ww=ww, M=M, K=K, N=N, off=off))
        xp = (rng.standard_normal((M, K + 4)) * np.exp2(rng.integers(-6, 7, size=(M, 1)))).astype(np.float32)
        wt = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
        fa, fb = mx.fmt(block, wx), mx.fmt(block, ww)
        B = mx.quantize_pack(T.dev(wt), fb, mx.MX_LAYOUT_FRAGMENT)
        scratch = mx.linear_workspace(M, K, N, fa, fb, T.DEV)
        y = torch.full((M, N), 3.0, dtype=torch.float32, device=T.DEV)
        xv = T.dev(xp)[:, off:off + K]
        mx.mx_linear(xv, M, K, K + 4, fa, scratch, B, N, fb, mx.MX_LAYOUT_FRAGMENT, y, N)
        torch.cuda.synchronize()
        y_ref, mag = orc.linear(xp[:, off:off + K], wt, block, wx, ww, want_mag=True)
        T.check_product(T.host(y), y_ref, mag, "random linear")


@pytest.mark.parametrize("seed", SEEDS)
def test_random_attention(seed):
    """mx_attention over sequence lengths, head dimensions, width draws, one- and two-row blocks."""
    rng = np.random.default_rng(1000 * seed + 3)
    for it in range(16):
        Sq = int(rng.integers(1, 200)); Sk = int(rng.integers(1, 20)) * 16; dim = int(rng.choice([16, 32, 48, 64, 96, 128]))
        widths = tuple(int(v) for v in rng.integers(2, 9, size=4)); R = int(rng.choice([1, 2]))
        if R == 2: Sq += Sq % 2
        say("attention", it, dict(Sq=Sq, Sk=Sk, dim=dim, widths=widths, R=R))
        Q = rng.standard_normal((2, Sq, dim)).astype(np.float32)
        K = rng.standard_normal((2, Sk, dim)).astype(np.float32)
        V = rng.standard_normal((2, Sk, dim)).astype(np.float32)
        r = T.run_attention(Q, K, V, widths, 0.9 * dim ** -0.5, block_rows=R, max_maybe=5e-2)
        say("   worst/bound", r)

@pytest.mark.parametrize("seed", SEEDS[:2])
def test_random_wide_exponents_fragment_layout(seed):
    """Fragment layout, block exponents over 60 binades, every row class (dot, stream, tiled kernels), with a block
    whose halves cancel sprinkled in: the plain criterion holds on any data there."""
    rng = np.random.default_rng(7000 + 10 * seed + 0)
    for it in range(60):
        block = int(rng.choice([16, 32, 64])); wa = int(rng.integers(2, 9)); wb = int(rng.integers(2, 9))
        M = int(rng.choice([1, 2, 3, 4, 7, 8, 9, 40, 130])); N = int(rng.integers(1, 300)); K = int(rng.integers(1, 24)) * block
        say("a", it, dict(block=block, wa=wa, wb=wb, M=M, N=N, K=K))
        qa, _ = T.random_operand(rng, M, K, block, wa, 0, 1); qb, _ = T.random_operand(rng, N, K, block, wb, 0, 1)
        base = rng.integers(60, 200, size=(1, K // block))
        ea = (base + rng.integers(-30, 31, size=(M, K // block))).clip(0, 255).astype(np.uint8)
        eb = (255 - base + rng.integers(-30, 31, size=(N, K // block))).clip(0, 255).astype(np.uint8)
        # sprinkle blocks whose halves cancel
        if K // block >= 2:
            blk = int(rng.integers(0, K // block))
            qa[:, blk * block:(blk + 1) * block] = 1
            qb[:, blk * block:blk * block + block // 2] = 1; qb[:, blk * block + block // 2:(blk + 1) * block] = -1
        A, fa = T.gpu_operand(qa, ea, block, wa); B, fb = T.gpu_operand(qb, eb, block, wb)
        y = mx.gemm(A, fa, B, fb, M, N, K); torch.cuda.synchronize()
        y_ref, mag = orc.gemm(qa, ea, wa, qb, eb, wb, block, want_mag=True)
        T.check_product(T.host(y)[0], y_ref, mag, "random wide exponents")


@pytest.mark.parametrize("seed", SEEDS[:2])
def test_random_fused_quantize_pack(seed):
    """mx_quantize_pack against mx_quantize + mx_pack (same bytes) on both layouts, one- and two-row blocks, batches;
    mx_unpack returns the oracle's canonical form."""
    rng = np.random.default_rng(7000 + 10 * seed + 1)
    for it in range(60):
        layout = int(rng.integers(0, 2)); block = int(rng.choice([16, 32, 64])); w = int(rng.integers(2, 9)); R = int(rng.choice([1, 1, 2]))
        rounding = int(rng.integers(0, 2)); batch = int(rng.choice([1, 2, 3])); rows = int(rng.integers(1, 200)); cols = int(rng.integers(1, 20)) * block
        if R == 2: rows += rows % 2
        say("b", it, dict(layout=layout, block=block, w=w, R=R, rounding=rounding, batch=batch, rows=rows, cols=cols))
        x = (rng.standard_normal((batch, rows, cols)) * np.exp2(rng.integers(-20, 20, size=(batch, rows, 1)))).astype(np.float32)
        x[rng.random(x.shape) < 0.03] = 0.0
        f = mx.fmt(block, w, 8, rounding, R)
        xd = T.dev(x)
        n = mx.mx_packed_bytes(batch, rows, cols, f, layout)
        p1 = torch.zeros(n, dtype=torch.uint8, device=T.DEV); p2 = torch.zeros(n, dtype=torch.uint8, device=T.DEV)
        mant, exps = mx.quantize(xd, f)
        mx.mx_pack(mant, exps, batch, rows, cols, f, layout, p1)
        mx.mx_quantize_pack(xd, batch, rows, cols, cols, rows * cols, f, layout, p2)
        um, ue = mx.unpack(p2, batch, rows, cols, f, layout)
        torch.cuda.synchronize()
        assert torch.equal(p1, p2)
        for b in range(batch):
            q, ex = orc.quantize(x[b], block, w, 8, rounding, block_rows=R)
            assert np.array_equal(T.host(um).reshape(batch, -1)[b], orc.pack_bits(q, w).reshape(-1))
            assert np.array_equal(T.host(ue).reshape(batch, -1)[b], ex.reshape(-1))


@pytest.mark.parametrize("seed", SEEDS[:2])
def test_random_minifloat(seed):
    """Block Minifloat / Block Logarithm quantizer over every (e, m) with 1 + e + m <= 8, bit-exact."""
    rng = np.random.default_rng(7000 + 10 * seed + 2)
    for it in range(60):
        block = int(rng.choice([8, 16, 32, 64])); e = int(rng.integers(1, 8)); m = int(rng.integers(0, 8 - e)); rounding = int(rng.integers(0, 2))
        rows = int(rng.integers(1, 100)); cols = int(rng.integers(1, 40)) * block
        say("c", it, dict(block=block, e=e, m=m, rounding=rounding, rows=rows, cols=cols))
        x = (rng.standard_normal((rows, cols)) * np.exp2(rng.integers(-30, 30, size=(rows, 1)))).astype(np.float32)
        x[rng.random(x.shape) < 0.03] = 0.0
        T.run_minifloat(x, block, e, m, rounding)


@pytest.mark.parametrize("seed", SEEDS[:2])
def test_random_cast(seed):
    """Width cast over width pairs, exponent widths, roundings, one- and two-row blocks, any column count."""
    rng = np.random.default_rng(7000 + 10 * seed + 3)
    for it in range(60):
        block = int(rng.choice([8, 16, 32, 64])); ws = int(rng.integers(2, 9)); wd = int(rng.integers(2, 9)); R = int(rng.choice([1, 1, 2]))
        es = int(rng.choice([8, 8, 5])); ed = int(rng.choice([8, 8, 4])); rounding = int(rng.integers(0, 2)); batch = int(rng.choice([1, 2]))
        rows = int(rng.integers(1, 60)); cols = int(rng.integers(1, 20)) * block
        if R == 2: rows += rows % 2
        say("d", it, dict(block=block, ws=ws, wd=wd, R=R, es=es, ed=ed, rounding=rounding, batch=batch, rows=rows, cols=cols))
        q = rng.integers(-(2 ** (ws - 1)), 2 ** (ws - 1), size=(batch, rows, cols)).astype(np.int8)
        q[:, :, ::3] //= 4
        ex = rng.integers(0, 2 ** es, size=(batch, rows // R, cols // block)).astype(np.uint8)
        T.check_cast(q, ex, block, ws, wd, es, ed, rounding, batch, R)

@pytest.mark.parametrize("seed", SEEDS[:2])
def test_random_fused_linear_layer(seed):
    """mx_gemm_q against mx_gemm, the bias add and mx_quantize_pack run one by one (same bytes): block sizes, one- and
    two-row blocks, widths, ragged M, batches, with and without bias."""
    rng = np.random.default_rng(9000 + 10 * seed + 0)
    MAT, DEV = T.MAT, T.DEV
    for it in range(30):
        block = int(rng.choice([16, 32, 64])); R = int(rng.choice([1, 2])); wx = int(rng.integers(2, 9)); ww = int(rng.integers(2, 5)); wo = int(rng.integers(2, 9))
        M = int(rng.integers(1, 300)); K = int(rng.integers(1, 12)) * 64; N = int(rng.integers(1, 12)) * 64; batch = int(rng.choice([1, 2]))
        if R == 2: M += M % 2
        with_bias = bool(rng.integers(0, 2))
        say("gemm_q", it, dict(block=block, R=R, wx=wx, ww=ww, wo=wo, M=M, K=K, N=N, batch=batch, bias=with_bias))
        x = rng.standard_normal((batch, M, K)).astype(np.float32)
        wt = (rng.standard_normal((batch, N, K)) * 0.02).astype(np.float32)
        bias = (rng.standard_normal(N) * 0.1).astype(np.float32)
        fa, fb = mx.fmt(block, wx, block_rows=R), mx.fmt(block, ww, block_rows=R)
        fbias, fo = mx.fmt(block, 4), mx.fmt(block, wo, block_rows=R)
        A = mx.quantize_pack(T.dev(x), fa, MAT); B = mx.quantize_pack(T.dev(wt), fb, MAT)
        bm, be = mx.quantize(T.dev(bias.reshape(1, N)), fbias)
        n_out = mx.mx_packed_bytes(batch, M, N, fo, MAT)
        out = torch.zeros(n_out, dtype=torch.uint8, device=DEV)
        st = mx.mx_gemm_q(batch, M, N, K, A, fa, B, fb, MAT, bm if with_bias else None, be if with_bias else None, fbias, fo, out, check=False)
        if st == mx.MX_ERR_UNSUPPORTED:
            say("   unsupported"); continue
        assert st == mx.MX_OK, st
        y = mx.gemm(A, fa, B, fb, M, N, K, batch=batch, layout=MAT)
        if with_bias: y = y + mx.dequantize(bm, be, 1, 1, N, fbias)[0]
        ref = torch.zeros(n_out, dtype=torch.uint8, device=DEV)
        mx.mx_quantize_pack(y.contiguous(), batch, M, N, N, M * N, fo, MAT, ref)
        torch.cuda.synchronize()
        assert torch.equal(out, ref)


@pytest.mark.parametrize("seed", SEEDS[:2])
def test_random_quantize_pack_down_the_columns(seed):
    """mx_quantize_pack_axis0 against the oracle's quantization of the transposed matrix: ragged shapes, row pitch,
    one- and two-row blocks, narrow exponents, batches."""
    rng = np.random.default_rng(9000 + 10 * seed + 1)
    MAT, DEV = T.MAT, T.DEV
    for it in range(40):
        rows = int(rng.integers(1, 40)) * 16; cols = int(rng.integers(1, 200)); w = int(rng.integers(2, 9)); R = int(rng.choice([1, 2])); rounding = int(rng.integers(0, 2))
        e = int(rng.choice([8, 8, 5])); batch = int(rng.choice([1, 3])); pad = int(rng.choice([0, 1, 4]))
        if R == 2: cols += cols % 2
        say("axis0", it, dict(rows=rows, cols=cols, w=w, R=R, rounding=rounding, e=e, batch=batch, pad=pad))
        x = (rng.standard_normal((batch, rows, cols + pad)) * np.exp2(rng.integers(-10, 10, size=(batch, 1, cols + pad)))).astype(np.float32)
        f = mx.fmt(16, w, e, rounding, R)
        xd = T.dev(x); xv = xd[:, :, :cols]
        got = torch.zeros((mx.mx_packed_bytes(batch, cols, rows, f, MAT),), dtype=torch.uint8, device=DEV)
        mx.mx_quantize_pack_axis0(xv, batch, rows, cols, cols + pad, rows * (cols + pad), f, MAT, got)
        um, ue = mx.unpack(got, batch, cols, rows, f, MAT)
        torch.cuda.synchronize()
        for b in range(batch):
            oq, oe = orc.quantize(np.ascontiguousarray(x[b, :, :cols].T), 16, w, e, rounding, block_rows=R)
            assert np.array_equal(T.host(um).reshape(batch, -1)[b], orc.pack_bits(oq, w).reshape(-1))
            assert np.array_equal(T.host(ue).reshape(batch, -1)[b], oe.reshape(-1))


@pytest.mark.parametrize("seed", SEEDS[:2])
def test_random_matrix_layout_products(seed):
    """Matrix-core layout on heavy-tailed activations and N(0, 0.02) weights (the workloads' structure): all block sizes
    and width pairs, ragged M, N, K, batches; the plain criterion."""
    rng = np.random.default_rng(9000 + 10 * seed + 2)
    MAT, DEV = T.MAT, T.DEV
    for it in range(40):
        block = int(rng.choice([16, 32, 64])); wa = int(rng.integers(2, 9)); wb = int(rng.integers(2, 9))
        M = int(rng.integers(1, 400)); N = int(rng.integers(1, 700)); K = int(rng.integers(1, 20)) * block; batch = int(rng.choice([1, 2]))
        say("matrix gemm", it, dict(block=block, wa=wa, wb=wb, M=M, N=N, K=K, batch=batch))
        x = (rng.standard_t(3, size=(batch, M, K))).astype(np.float32)
        wt = (rng.standard_normal((batch, N, K)) * 0.02).astype(np.float32)
        fa, fb = mx.fmt(block, wa), mx.fmt(block, wb)
        A = mx.quantize_pack(T.dev(x), fa, MAT); B = mx.quantize_pack(T.dev(wt), fb, MAT)
        y = mx.gemm(A, fa, B, fb, M, N, K, batch=batch, layout=MAT); torch.cuda.synchronize()
        for b in range(batch):
            y_ref, mag = orc.linear(x[b], wt[b], block, wa, wb, want_mag=True)
            T.check_product(T.host(y)[b], y_ref, mag, "matrix gemm")


@pytest.mark.parametrize("seed", SEEDS[:2])
def test_random_strided_inputs(seed):
    """Views with a row pitch, a batch pitch and an unaligned first element through mx_quantize (both axes, one- and
    two-row blocks) and, where the alignment allows, mx_quantize_pack on both layouts."""
    rng = np.random.default_rng(11000 + seed)
    DEV = T.DEV
    for it in range(80):
        block = int(rng.choice([8, 16, 32, 64])); w = int(rng.integers(2, 9)); R = int(rng.choice([1, 1, 2])); axis = int(rng.integers(0, 2))
        rounding = int(rng.integers(0, 2)); batch = int(rng.choice([1, 2, 3]))
        padc = int(rng.choice([0, 1, 3, 4, 8])); padr = int(rng.choice([0, 1, 2])); off = int(rng.choice([0, 0, 1, 2, 4]))
        nb = int(rng.integers(1, 24))
        if axis == 1:
            rows, cols = int(rng.integers(1, 150)), nb * block
            if R == 2: rows += rows % 2
        else:
            rows, cols = nb * block, int(rng.integers(1, 150))
            if R == 2: cols += cols % 2
        say("quantize", it, dict(block=block, w=w, R=R, axis=axis, rounding=rounding, batch=batch, rows=rows, cols=cols, padc=padc, padr=padr, off=off))
        big = (rng.standard_normal((batch, rows + padr, cols + padc + off)) * np.exp2(rng.integers(-12, 12, size=(batch, rows + padr, 1)))).astype(np.float32)
        bd = T.dev(big)
        xv = bd[:, :rows, off:off + cols]
        f = mx.fmt(block, w, 8, rounding, R)
        mant, exps = mx.quantize(xv, f, axis=axis)
        torch.cuda.synchronize()
        for b in range(batch):
            xo = big[b, :rows, off:off + cols]
            xo = np.ascontiguousarray(xo if axis == 1 else xo.T)
            q, ex = orc.quantize(xo, block, w, 8, rounding, block_rows=R)
            assert np.array_equal(T.host(exps).reshape(batch, -1)[b], ex.reshape(-1)), "exps"
            assert np.array_equal(T.host(mant).reshape(batch, -1)[b], orc.pack_bits(q, w).reshape(-1)), "mant"
        # the fused quantize+pack on the same view (blocks of 16/32/64 only; the matrix layout wants 16-byte aligned rows)
        if axis == 1 and block >= 16:
            for layout in (0, 1):
                n = mx.mx_packed_bytes(batch, rows, cols, f, layout)
                p = torch.zeros(n, dtype=torch.uint8, device=DEV)
                st = mx.mx_quantize_pack(xv, batch, rows, cols, xv.stride(1), xv.stride(0), f, layout, p, check=False)
                if st == mx.MX_ERR_UNSUPPORTED:
                    say("   layout", layout, "unsupported (alignment)"); continue
                assert st == mx.MX_OK, st
                um, ue = mx.unpack(p, batch, rows, cols, f, layout)
                torch.cuda.synchronize()
                assert torch.equal(um, mant) and torch.equal(ue, exps), ("fused", layout)


@pytest.mark.parametrize("seed", SEEDS[:2])
def test_random_dequantize_and_round_trips(seed):
    """mx_dequantize on arbitrary codes and exponent bytes (exact inside the fp32 range, infinity beyond it), and
    mx_pack / mx_unpack round trips on arbitrary bytes for both layouts, one- and two-row blocks."""
    rng = np.random.default_rng(13000 + seed)
    for it in range(80):
        block = int(rng.choice([8, 16, 32, 64])); w = int(rng.integers(2, 9)); e = int(rng.choice([8, 8, 6, 3])); R = int(rng.choice([1, 2]))
        batch = int(rng.choice([1, 2])); rows = int(rng.integers(1, 120)); cols = int(rng.integers(1, 24)) * block
        if R == 2: rows += rows % 2
        say("dequantize", it, dict(block=block, w=w, e=e, R=R, batch=batch, rows=rows, cols=cols))
        q = rng.integers(-(2 ** (w - 1)), 2 ** (w - 1), size=(batch, rows, cols)).astype(np.int8)
        ex = rng.integers(0, 2 ** e, size=(batch, rows // R, cols // block)).astype(np.uint8)
        f = mx.fmt(block, w, e, block_rows=R)
        mant = T.dev(orc.pack_bits(q.reshape(-1, cols), w).reshape(-1))
        y = T.host(mx.dequantize(mant, T.dev(ex.reshape(-1)), batch, rows, cols, f)).astype(np.float64)
        for b in range(batch):
            want = orc.dequantize(q[b], orc.row_exps(ex[b], R), block, w, e)
            big = np.abs(want) > 3.4028234663852886e38                  # beyond fp32: the device gives infinity
            ok = (y[b] == want) | (np.abs(want) < 2.0 ** -126) | big    # exact unless below the fp32 normal range
            assert ok.all(), ("dequantize", np.argwhere(~ok)[:5].tolist())
            assert np.all((np.abs(y[b] - want) <= 2.0 ** -149) | big)
            assert np.all(np.isinf(y[b][big]))
        if block >= 16:
            for layout in (0, 1):
                lo, hi = (0, 256)
                if layout == 1: lo, hi = ((w - 1, 254) if block == 16 else (0, 251))
                ex2 = rng.integers(lo, hi, size=(batch, rows // R, cols // block)).astype(np.uint8)
                f8 = mx.fmt(block, w, 8, block_rows=R)
                p = mx.pack(mant, T.dev(ex2.reshape(-1)), batch, rows, cols, f8, layout)
                m2, e2 = mx.unpack(p, batch, rows, cols, f8, layout)
                torch.cuda.synchronize()
                assert torch.equal(m2, mant) and np.array_equal(T.host(e2), ex2.reshape(-1)), ("roundtrip", layout)
