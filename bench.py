#!/usr/bin/env python3
"""Benchmark of the MXInt hot path on one MI355X.

One step = one pass of the whole path over the LLaMA-7B-shaped prefill linears (M = 2048 tokens;
4096x4096, 4096x11008, 11008x4096; block 32, activations 8 bits, weights 4 bits): for each linear,
mx_quantize of the fp32 activations, mx_pack, mx_gemm against the pre-packed weights.  All inputs
are seeded synthetic tensors already resident in HBM.  The step's value is 2*M*N*K summed over the
three linears divided by the wall time of the step (quantizer and pack included).

Besides the contract fields the JSON line carries
  roofline      the product kernel: algorithmic 2*M*N*K per launch / average launch duration
                (HIP events around every mx_gemm of the timed region) against the int8 MFMA peak;
  kernels       HBM-bound kernels timed on their own over rings of distinct buffers larger than the
                last-level cache: the quantizer (GB/s) and the decode linear (LLaMA-13B shapes);
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
INT8_MFMA_PEAK_TOPS = 5000.0


def recorded_traffic():
    """HBM-side bytes per mx_gemm launch from the committed rocprofv3 counter summary, or None when the
    product kernel's source has changed since the counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "mx_gemm_llama7b_prefill_traffic.txt")
    try:
        fields = {}
        for line in open(path):
            if ":" in line and line.startswith("  "):
                k, v = line.strip().split(":", 1)
                fields[k.strip()] = v.strip()
        h = hashlib.sha256()
        for rel in ("paper_2307_15517_amd/csrc/mx_gemm_scaled.hip", "paper_2307_15517_amd/csrc/mx_matrix.h"):
            h.update(open(os.path.join(ROOT, rel), "rb").read())
        if fields.get("source_sha256") != h.hexdigest():
            return None
        return int(fields["traffic_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernels", action="store_true", help="skip the separate quantizer / decode timings")
    ap.add_argument("--layout", choices=["matrix", "fragment"], default="matrix",
                    help="operand layout of the prefill product: block-scaled matrix cores (default) or int8 MFMA")
    ap.add_argument("--unfused", action="store_true", help="mx_quantize + mx_pack instead of mx_quantize_pack")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (known traffic, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (--gpus 1); the path has no multi-GPU part",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2307_15517_amd import inputs, mx

    mx.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    L = mx.MX_LAYOUT_MATRIX if args.layout == "matrix" else mx.MX_LAYOUT_FRAGMENT
    LF = mx.MX_LAYOUT_FRAGMENT

    # ---------------------------------------------------------------- workload: LLaMA-7B prefill linears
    cases = inputs.llama7b_prefill()
    ring = 6                      # distinct activation buffers per linear: 6 * (33.5 + 33.5 + 90) MB > 256 MB cache
    work = []
    for case in cases:
        x, wt = inputs.make(case)
        fa, fb = mx.fmt(case.block, case.wx), mx.fmt(case.block, case.ww)
        wd = torch.from_numpy(wt).to(dev)
        bm, be = mx.quantize(wd, fb)
        B = mx.pack(bm, be, 1, case.N, case.K, fb, L)
        del wd, bm, be
        xs = [torch.from_numpy(x).to(dev)]
        for r in range(1, ring):
            xs.append(torch.roll(xs[0], shifts=r, dims=0).contiguous())
        w = dict(case=case, fa=fa, fb=fb, B=B, xs=xs,
                 mant=torch.empty(mx.mx_mant_bytes(1, case.M, case.K, fa), dtype=torch.uint8, device=dev),
                 exps=torch.empty(mx.mx_exps_bytes(1, case.M, case.K, fa), dtype=torch.uint8, device=dev),
                 A=torch.empty(mx.mx_packed_bytes(1, case.M, case.K, fa, L), dtype=torch.uint8, device=dev),
                 Y=[torch.empty((case.M, case.N), dtype=torch.float32, device=dev) for _ in range(2)],
                 ops=2.0 * case.M * case.N * case.K)
        work.append(w)
    total_ops = sum(w["ops"] for w in work)
    gemm_events = []

    def step(i, timed):
        for w in work:
            c = w["case"]
            x = w["xs"][i % ring]
            if args.unfused:
                mx.mx_quantize(x, 1, c.M, c.K, c.K, 0, 1, w["fa"], w["mant"], w["exps"])
                mx.mx_pack(w["mant"], w["exps"], 1, c.M, c.K, w["fa"], L, w["A"])
            else:
                mx.mx_quantize_pack(x, 1, c.M, c.K, c.K, 0, w["fa"], L, w["A"])
            if timed:
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
            mx.mx_gemm(1, c.M, c.N, c.K, w["A"], w["fa"], w["B"], w["fb"], L, w["Y"][i % 2], c.N, 0)
            if timed:
                e1.record()
                gemm_events.append((e0, e1, w["ops"]))

    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec = t1 - t0
    ms_per_step = 1e3 * sec / args.steps
    value = total_ops * args.steps / sec / 1e12

    gemm_ms = sum(e0.elapsed_time(e1) for e0, e1, _ in gemm_events)
    gemm_ops = sum(o for _, _, o in gemm_events)
    achieved = gemm_ops / (gemm_ms * 1e-3) / 1e12
    kname = ("mx_gemm (block-scaled fp6 MFMA, two mantissa pieces for 8-bit activations)" if args.layout == "matrix"
             else "mx_gemm (int8 MFMA, block-exponent epilogue)")
    roofline = {"kernel": kname, "bound": "mfma",
                "achieved": round(achieved, 2), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                "frac": round(achieved / INT8_MFMA_PEAK_TOPS, 4),
                "traffic": recorded_traffic() if args.layout == "matrix" else None,
                "avg_launch_ms": round(gemm_ms / len(gemm_events), 4)}

    # ---------------------------------------------------------------- HBM-bound kernels on their own
    kernels = {}
    if not args.no_kernels:
        def time_launches(fn, n, reps=3):
            best = None
            for _ in range(reps):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(n):
                    fn(i)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / n
                best = ms if best is None else min(best, ms)
            return best

        # quantizer: 4 bytes read + w/8 + 1/block bytes written per element, over a ring of distinct inputs
        # (> 1 GB in all) so that nothing is served from the last-level cache
        for w in (work[0], work[2]):
            c = w["case"]
            nring = int(1.3e9 // (c.M * c.K * 4)) + 1
            qring = [torch.randn((c.M, c.K), dtype=torch.float32, device=dev) for _ in range(nring)]
            ms = time_launches(lambda i: mx.mx_quantize(qring[i % nring], 1, c.M, c.K, c.K, 0, 1, w["fa"],
                                                        w["mant"], w["exps"]), 2 * nring)
            qbytes = c.M * c.K * (4 + c.wx / 8 + 1 / c.block)
            kernels["quantize_%dx%d_w%d_b%d" % (c.M, c.K, c.wx, c.block)] = {
                "GBps": round(qbytes / ms / 1e6, 1), "frac_hbm": round(qbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                "us": round(ms * 1e3, 2), "bytes": int(qbytes)}
            if c.K == 11008:
                # the paper's own block shape: 16 columns x 2 rows per exponent, MXInt((16,2),8,7)
                f2 = mx.fmt(16, 8, block_rows=2)
                e2 = torch.empty(mx.mx_exps_bytes(1, c.M, c.K, f2), dtype=torch.uint8, device=dev)
                ms = time_launches(lambda i: mx.mx_quantize(qring[i % nring], 1, c.M, c.K, c.K, 0, 1, f2,
                                                            w["mant"], e2), 2 * nring)
                kernels["quantize_%dx%d_w8_b16x2" % (c.M, c.K)] = {
                    "GBps": round(qbytes / ms / 1e6, 1), "frac_hbm": round(qbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                    "us": round(ms * 1e3, 2), "bytes": int(qbytes)}
            if c.K == 11008:
                # the paper's other block formats at the same shape: Block Minifloat (1 + 4 + 3 bits) and Block
                # Logarithm (1 + 7 bits), one byte per element + one shared byte per block
                mcodes = torch.empty(c.M * c.K, dtype=torch.uint8, device=dev)
                mshared = torch.empty(c.M * c.K // c.block, dtype=torch.uint8, device=dev)
                for name, fm in (("bmf_e4m3", mx.mx_minifloat_format(c.block, 4, 3, mx.MX_RNE)),
                                 ("bl_e7", mx.mx_minifloat_format(c.block, 7, 0, mx.MX_RNE))):
                    ms = time_launches(lambda i: mx.mx_quantize_minifloat(qring[i % nring], 1, c.M, c.K, c.K, 0, fm,
                                                                          mcodes, mshared), 2 * nring)
                    mbytes = c.M * c.K * (4 + 1 + 1 / c.block)
                    kernels["quantize_%s_%dx%d_b%d" % (name, c.M, c.K, c.block)] = {
                        "GBps": round(mbytes / ms / 1e6, 1), "frac_hbm": round(mbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                        "us": round(ms * 1e3, 2), "bytes": int(mbytes)}
            if args.layout == "matrix":
                ms = time_launches(lambda i: mx.mx_quantize_pack(qring[i % nring], 1, c.M, c.K, c.K, 0, w["fa"], L,
                                                                 w["A"]), 2 * nring)
                pbytes = c.M * c.K * 4 + mx.mx_packed_bytes(1, c.M, c.K, w["fa"], L)
                kernels["quantize_pack_matrix_%dx%d_w%d_b%d" % (c.M, c.K, c.wx, c.block)] = {
                    "GBps": round(pbytes / ms / 1e6, 1), "frac_hbm": round(pbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                    "us": round(ms * 1e3, 2), "bytes": int(pbytes)}
            del qring
        # width cast inside the format, 8 -> 4 bits at the prefill activation shape:
        # (8 + 4)/8 + 2/block bytes per element
        c = work[2]["case"]
        f4 = mx.fmt(c.block, 4)
        nring = int(1.3e9 // (c.M * c.K)) + 1
        m8s = [torch.randint(0, 256, (c.M * c.K,), dtype=torch.uint8, device=dev) for _ in range(nring)]
        e8 = torch.randint(100, 140, (c.M * c.K // c.block,), dtype=torch.uint8, device=dev)
        m4 = torch.empty(mx.mx_mant_bytes(1, c.M, c.K, f4), dtype=torch.uint8, device=dev)
        e4 = torch.empty(mx.mx_exps_bytes(1, c.M, c.K, f4), dtype=torch.uint8, device=dev)
        calls = [mx.bound("mx_cast", m, e8, 1, c.M, c.K, work[2]["fa"], f4, m4, e4) for m in m8s]
        ms = time_launches(lambda i: calls[i % nring](), 2 * nring)
        cbytes = c.M * c.K * (1.5 + 2 / c.block)
        kernels["cast_%dx%d_w8_to_w4_b%d" % (c.M, c.K, c.block)] = {
            "GBps": round(cbytes / ms / 1e6, 1), "frac_hbm": round(cbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
            "us": round(ms * 1e3, 2), "bytes": int(cbytes)}
        del m8s, calls
        # the whole emulated linear layer (product + MXInt bias + output quantizer) in one kernel, against the
        # product followed by a separate quantize+pack of its fp32 result; 8-bit activations in and out, 4-bit
        # weights and bias: the three prefill linears (block 32) and the first one at block 16
        if args.layout == "matrix":
            for w, blk in [(work[0], 32), (work[1], 32), (work[2], 32), (work[0], 16)]:
                c = w["case"]
                fa_, fb_, fo_, fbias_ = mx.fmt(blk, 8), mx.fmt(blk, 4), mx.fmt(blk, 8), mx.fmt(blk, 4)
                if blk == 32:
                    A_, B_ = w["A"], w["B"]
                else:
                    A_ = mx.quantize_pack(w["xs"][0], fa_, L)
                    B_ = mx.quantize_pack(torch.randn((c.N, c.K), dtype=torch.float32, device=dev) * 0.02, fb_, L)
                bm_, be_ = mx.quantize(torch.randn((1, c.N), dtype=torch.float32, device=dev), fbias_)
                o_ = torch.empty(mx.mx_packed_bytes(1, c.M, c.N, fo_, L), dtype=torch.uint8, device=dev)
                y_ = w["Y"][0]
                fused = mx.bound("mx_gemm_q", 1, c.M, c.N, c.K, A_, fa_, B_, fb_, L, bm_, be_, fbias_, fo_, o_)
                plain = mx.bound("mx_gemm", 1, c.M, c.N, c.K, A_, fa_, B_, fb_, L, y_, c.N, 0)
                requant = mx.bound("mx_quantize_pack", y_, 1, c.M, c.N, c.N, 0, fo_, L, o_)
                ms_f = time_launches(lambda i: fused(), 20)
                ms_pq = time_launches(lambda i: (plain(), requant()), 20)
                kernels["linear_q_%dx%dx%d_b%d" % (c.M, c.N, c.K, blk)] = {
                    "fused_us": round(ms_f * 1e3, 2), "fused_TOPS": round(w["ops"] / ms_f / 1e9, 1),
                    "gemm_then_quantize_pack_us": round(ms_pq * 1e3, 2)}
                del o_
        # decode linear, LLaMA-13B shapes: 0.5625*N*K + 4*M*K + 4*M*N bytes per call
        for M in (1, 4, 8):
            for dc in inputs.llama13b_decode(M):
                fa, fb = mx.fmt(dc.block, dc.wx), mx.fmt(dc.block, dc.ww)
                x, wt = inputs.make(dc)
                wd = torch.from_numpy(wt).to(dev)
                bm, be = mx.quantize(wd, fb)
                B0 = mx.pack(bm, be, 1, dc.N, dc.K, fb, LF)
                nring = max(2, int(1.3e9 // B0.numel()))
                Bs = [B0] + [B0.clone() for _ in range(nring - 1)]
                xd = torch.from_numpy(x).to(dev)
                scratch = mx.linear_workspace(M, dc.K, dc.N, fa, fb, dev)
                y = torch.empty((M, dc.N), dtype=torch.float32, device=dev)
                calls = [mx.bound("mx_linear", xd, M, dc.K, dc.K, fa, scratch, Bw, dc.N, fb, LF, y, dc.N) for Bw in Bs]
                ms = time_launches(lambda i: calls[i % nring](), 2 * nring)
                nbytes = 0.5625 * dc.N * dc.K + 4 * M * dc.K + 4 * M * dc.N
                kernels["linear_%s_M%d" % (dc.name, M)] = {
                    "GBps": round(nbytes / ms / 1e6, 1), "frac_hbm": round(nbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                    "us": round(ms * 1e3, 2), "bytes": int(nbytes)}
                del Bs, B0, wd, bm, be

        # mixed-precision attention, 32 heads x 2048 positions x 128: both products are bound by the fp32
        # score matrix (written by Q K^T, read again to quantize P); algorithmic bytes per step below
        heads, seq, dim, ablock = 32, 2048, 128, 16
        LA = L          # block 16 on the matrix layout is the bfloat16 form; --layout fragment times the int8 path
        wq, wk, wp, wv = inputs.attention_widths(0)
        Qh, Kh, Vh = inputs.attention_qkv(0, heads, seq, dim)
        fq, fk, fpp, fv = (mx.fmt(ablock, w_) for w_ in (wq, wk, wp, wv))
        Qd, Kd, Vd = (torch.from_numpy(t).to(dev) for t in (Qh, Kh, Vh))
        pb = lambda r, c_, f_: mx.mx_packed_bytes(heads, r, c_, f_, LA)
        Aq = torch.empty(pb(seq, dim, fq), dtype=torch.uint8, device=dev)
        Bk = torch.empty(pb(seq, dim, fk), dtype=torch.uint8, device=dev)
        Ap = torch.empty(pb(seq, seq, fpp), dtype=torch.uint8, device=dev)
        Bv = torch.empty(pb(dim, seq, fv), dtype=torch.uint8, device=dev)
        vmant = torch.empty(mx.mx_mant_bytes(heads, dim, seq, fv), dtype=torch.uint8, device=dev)
        vexps = torch.empty(mx.mx_exps_bytes(heads, dim, seq, fv), dtype=torch.uint8, device=dev)
        Ss = [torch.empty((heads, seq, seq), dtype=torch.float32, device=dev) for _ in range(2)]
        Od = torch.empty((heads, seq, dim), dtype=torch.float32, device=dev)
        mx.mx_quantize_pack(Qd, heads, seq, dim, dim, seq * dim, fq, LA, Aq)
        mx.mx_quantize_pack(Kd, heads, seq, dim, dim, seq * dim, fk, LA, Bk)
        mx.mx_gemm(heads, seq, seq, dim, Aq, fq, Bk, fk, LA, Ss[0], seq, seq * seq)
        Ps = [torch.softmax(Ss[0] / dim ** 0.5, dim=-1).contiguous()]
        Ps.append(Ps[0].flip(0).contiguous())
        dens = lambda f_: f_.mant_bits / 8 + 1 / f_.block

        def attn_entry(name, ms, nbytes, ops=None):
            e = {"GBps": round(nbytes / ms / 1e6, 1), "frac_hbm": round(nbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                 "us": round(ms * 1e3, 2), "bytes": int(nbytes)}
            if ops:
                e["TOPS"] = round(ops / ms / 1e9, 1)
            kernels["attention_w%d%d%d%d_%s" % (wq, wk, wp, wv, name)] = e

        n_el = heads * seq * dim
        ms = time_launches(lambda i: mx.mx_quantize_pack(Qd, heads, seq, dim, dim, seq * dim, fq, LA, Aq), 20)
        attn_entry("quantize_pack_q", ms, n_el * 4 + Aq.numel())
        ms = time_launches(lambda i: mx.mx_gemm(heads, seq, seq, dim, Aq, fq, Bk, fk, LA, Ss[i % 2], seq, seq * seq), 10)
        attn_entry("scores_gemm", ms, Aq.numel() + Bk.numel() + 4 * heads * seq * seq, 2.0 * heads * seq * seq * dim)
        ms = time_launches(lambda i: mx.mx_quantize_pack(Ps[i % 2], heads, seq, seq, seq, seq * seq, fpp, LA, Ap), 10)
        attn_entry("quantize_pack_p", ms, 4 * heads * seq * seq + Ap.numel())
        ms = time_launches(lambda i: mx.mx_quantize(Vd, heads, seq, dim, dim, seq * dim, 0, fv, vmant, vexps), 20)
        attn_entry("quantize_v_along_seq", ms, n_el * (4 + dens(fv)))
        mx.mx_pack(vmant, vexps, heads, dim, seq, fv, LA, Bv)
        if LA == mx.MX_LAYOUT_MATRIX:
            ms = time_launches(lambda i: mx.mx_quantize_pack_axis0(Vd, heads, seq, dim, dim, seq * dim, fv, LA, Bv), 20)
            attn_entry("quantize_pack_v_along_seq", ms, n_el * 4 + Bv.numel())
        ms = time_launches(lambda i: mx.mx_gemm(heads, seq, dim, seq, Ap, fpp, Bv, fv, LA, Od, dim, seq * dim), 10)
        attn_entry("output_gemm", ms, Ap.numel() + Bv.numel() + 4 * n_el, 2.0 * heads * seq * seq * dim)
        del Ss, Ps, Ap
        # the same from packed Q, K, V^T to O in one kernel (scores and probabilities stay on chip); the
        # operation count is that of the two products of the definition
        if LA == mx.MX_LAYOUT_MATRIX:
            Ods = [torch.empty((heads, seq, dim), dtype=torch.float32, device=dev) for _ in range(2)]
            ms = time_launches(lambda i: mx.mx_attention(heads, seq, seq, dim, Aq, fq, Bk, fk, Bv, fv, fpp, dim ** -0.5,
                                                         LA, Ods[i % 2], dim, seq * dim), 10)
            attn_entry("fused_scores_softmax_quantize_output", ms, Aq.numel() + Bk.numel() + Bv.numel() + 4 * n_el,
                       4.0 * heads * seq * seq * dim)

            def whole(i):                               # from fp32 Q, K, V to fp32 O: four launches
                mx.mx_quantize_pack(Qd, heads, seq, dim, dim, seq * dim, fq, LA, Aq)
                mx.mx_quantize_pack(Kd, heads, seq, dim, dim, seq * dim, fk, LA, Bk)
                mx.mx_quantize_pack_axis0(Vd, heads, seq, dim, dim, seq * dim, fv, LA, Bv)
                mx.mx_attention(heads, seq, seq, dim, Aq, fq, Bk, fk, Bv, fv, fpp, dim ** -0.5, LA, Ods[i % 2], dim,
                                seq * dim)
            ms = time_launches(whole, 10)
            attn_entry("from_fp32_qkv_to_output", ms, 4 * 4 * n_el, 4.0 * heads * seq * seq * dim)

    # ---------------------------------------------------------------- the oracle on the host cores
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import mx_oracle as orc
        threads = orc.set_threads(0)
        # one whole step of the workload: every activation row of the three linears (a few seconds per
        # linear on the machine's cores); inputs are generated before the clock starts
        data = [(case,) + tuple(inputs.make(case)) for case in cases]
        t0 = time.perf_counter()
        for case, x, wt in data:
            qa, ea = orc.quantize(x, case.block, case.wx)
            qb, eb = orc.quantize(wt, case.block, case.ww)
            orc.gemm(qa, ea, case.wx, qb, eb, case.ww, case.block)
        dt = time.perf_counter() - t0
        # the same code on one thread, on the first 64 activation rows of the first linear (product only scales
        # with the rows; the weights are quantized once more)
        case, x, wt = data[0]
        orc.set_threads(1)
        t1 = time.perf_counter()
        qa, ea = orc.quantize(x[:64], case.block, case.wx)
        qb, eb = orc.quantize(wt, case.block, case.ww)
        orc.gemm(qa, ea, case.wx, qb, eb, case.ww, case.block)
        dt1 = time.perf_counter() - t1
        orc.set_threads(threads)
        single = {"value": round(2.0 * 64 * case.N * case.K / dt1 / 1e12, 6), "unit": "TOP/s", "cores": 1,
                  "seconds": round(dt1, 2), "sample": "64 activation rows of %s" % case.name}
        cpu = {"value": round(total_ops / dt / 1e12, 5), "unit": "TOP/s", "cores": threads, "single_thread": single,
               "kind": "oracle", "seconds": round(dt, 2),
               "sample": "one step of the workload: for each of %s quantize all %d activation rows and all weights, "
                         "then the product (%.1f GOP in all); C oracle with OpenMP over rows"
                         % (", ".join(c.name for c in cases), cases[0].M, total_ops / 1e9)}

    out = {
        "metric": "MXInt GEMM TOPS + quantize/GEMV GB/s (% roofline) at LLaMA-7B linear shapes",
        "value": round(value, 2), "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "fp6(exact int pieces)+fp32 acc" if args.layout == "matrix" else "int8",
        "data": "synthetic",
        "config": {"workload": "llama7b_prefill_M2048: quantize+pack+gemm over 4096x4096, 4096x11008, "
                               "11008x4096; block 32, act 8 bits, weight 4 bits"},
        "roofline": roofline, "kernels": kernels, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
