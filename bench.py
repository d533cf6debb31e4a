#!/usr/bin/env python3
"""Benchmark of the MXInt hot path on one MI355X.

One step = one pass of the whole path over the LLaMA-7B-shaped prefill linears (M = 2048 tokens;
4096x4096, 4096x11008, 11008x4096; block 32, activations 8 bits, weights 4 bits): for each linear,
mx_quantize of the fp32 activations, mx_pack, mx_gemm against the pre-packed weights.  All inputs
are seeded synthetic tensors already resident in HBM.  The step's value is 2*M*N*K summed over the
three linears divided by the wall time of the step (quantizer and pack included).

Besides the contract fields the JSON line carries
  roofline      the product kernel: algorithmic 2*M*N*K per launch / average launch duration against the int8
                MFMA peak; the durations come from a second run of the same K steps with a HIP event on either
                side of every mx_gemm (the timed steps themselves carry no events: each one stalls the stream
                for a few microseconds);
                "achievable": what a bare loop of matrix instructions reaches on this GPU (zeros and random
                operands, with the shader clock each ran at) and what streaming kernels reach;
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
MIN_LAUNCHES = 200            # launches behind every per-kernel figure


class HipEvents:
    """HIP events created without the system-scope fence (hipEventDisableSystemFence): recording one then costs the
    stream a marker, not a flush of the caches towards the host, so a pair brackets the kernel between them and little
    else.  Recorded on the stream the kernels are launched on."""
    DISABLE_SYSTEM_FENCE = 0x20000000

    def __init__(self, n, stream_handle):
        import ctypes
        self.ct = ctypes
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.stream = ctypes.c_void_p(stream_handle)
        self.events = []
        for _ in range(n):
            e = ctypes.c_void_p()
            if self.hip.hipEventCreateWithFlags(ctypes.byref(e), self.DISABLE_SYSTEM_FENCE) != 0:
                raise RuntimeError("hipEventCreateWithFlags failed")
            self.events.append(e)

    def record(self, i):
        if self.hip.hipEventRecord(self.events[i], self.stream) != 0:
            raise RuntimeError("hipEventRecord failed")

    def elapsed_ms(self, i, j):
        ms = self.ct.c_float()
        if self.hip.hipEventElapsedTime(self.ct.byref(ms), self.events[i], self.events[j]) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return float(ms.value)

    def destroy(self):
        for e in self.events:
            self.hip.hipEventDestroy(e)
        self.events = []


class Probes:
    """ctypes front end of libmx_probes.so (csrc/probes/mx_probes.hip): bare streaming kernels and bare loops of
    matrix instructions, the denominators a kernel can be held against on this GPU besides the published peaks."""

    def __init__(self, torch, dev):
        import ctypes
        path = os.path.join(ROOT, "paper_2307_15517_amd", "libmx_probes.so")
        if not os.path.exists(path):
            raise FileNotFoundError("%s is missing: build it with `python -m paper_2307_15517_amd.build`" % path)
        self.lib = ctypes.CDLL(path)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        self.lib.mxp_read.argtypes = [vp, sz, vp, vp]
        self.lib.mxp_write.argtypes = [vp, sz, vp]
        self.lib.mxp_copy.argtypes = [vp, vp, sz, vp]
        self.lib.mxp_mfma_fp6.argtypes = [vp, vp, i32, vp, vp, vp]
        self.lib.mxp_mfma_i8.argtypes = [vp, vp, i32, vp, vp, vp]
        self.lib.mxp_mfma_waves.restype = i32
        self.torch, self.dev, self.ctypes = torch, dev, ctypes
        self.stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        self.sink = torch.zeros(16, dtype=torch.float32, device=dev)
        self.pool = None
        self._floors = {}

    def _pool(self):
        if self.pool is None:           # 1.5 GB touched once: rings of distinct buffers are slices of it
            self.pool = self.torch.ones(1536 << 20, dtype=self.torch.uint8, device=self.dev)
        return self.pool

    def stream_ms(self, kind, nbytes, timer):
        """Median time of one streaming pass (read / write / copy of nbytes) over a ring of distinct buffers
        larger than the last-level cache."""
        key = (kind, int(nbytes))
        if key in self._floors:
            return self._floors[key]
        nbytes = int(nbytes) // 256 * 256
        pool = self._pool()
        span = nbytes * (2 if kind == "copy" else 1)
        if span > pool.numel():
            raise ValueError("stream probe of %d bytes does not fit the %d-byte pool" % (span, pool.numel()))
        nring = max(1, min(64, int(min(1.3e9, pool.numel()) // span)))     # every buffer of the ring lies inside the pool
        assert nring * span <= pool.numel()
        base = pool.data_ptr()
        vp = self.ctypes.c_void_p
        calls = []
        for r in range(nring):
            a = base + r * span
            if kind == "read":
                calls.append((self.lib.mxp_read, (vp(a), nbytes, vp(self.sink.data_ptr()), self.stream)))
            elif kind == "write":
                calls.append((self.lib.mxp_write, (vp(a), nbytes, self.stream)))
            else:
                calls.append((self.lib.mxp_copy, (vp(a + nbytes), vp(a), nbytes, self.stream)))

        def fn(i):
            f, a = calls[i % nring]
            assert f(*a) == 0
        ms = timer(fn, 2 * nring)
        self._floors[key] = ms
        return ms

    def mfma(self, kind, pattern, iters=20000):
        """TOP/s and shader clock of a bare loop of matrix instructions: kind "fp6" (block-scaled 6-bit floats,
        32x32x64) or "i8" (32x32x32), operands all zero or random bits."""
        torch = self.torch
        ndw = 64 * 4 * (8 if kind == "fp6" else 4)
        if pattern == "zeros":
            a = torch.zeros(ndw, dtype=torch.int32, device=self.dev)
            b = torch.zeros(ndw, dtype=torch.int32, device=self.dev)
        else:
            g = torch.Generator(device=self.dev)
            g.manual_seed(7)
            a = torch.randint(-2 ** 31, 2 ** 31 - 1, (ndw,), dtype=torch.int32, device=self.dev, generator=g)
            b = torch.randint(-2 ** 31, 2 ** 31 - 1, (ndw,), dtype=torch.int32, device=self.dev, generator=g)
        waves = self.lib.mxp_mfma_waves()
        out = torch.zeros((waves, 2), dtype=torch.int64, device=self.dev)
        fn = self.lib.mxp_mfma_fp6 if kind == "fp6" else self.lib.mxp_mfma_i8
        vp = self.ctypes.c_void_p
        args = (vp(a.data_ptr()), vp(b.data_ptr()), iters, vp(out.data_ptr()), vp(self.sink.data_ptr()), self.stream)
        assert fn(*args) == 0                                   # warm-up
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            assert fn(*args) == 0
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 3
        ops = waves * iters * 16 * 2.0 * 32 * 32 * (64 if kind == "fp6" else 32)
        o = out.cpu().numpy().astype("float64")
        ghz = float(__import__("numpy").median(o[:, 0] / o[:, 1])) * 0.1          # cycles per 10 ns tick
        return {"TOPS": round(ops / ms / 1e9, 1), "shader_clock_GHz": round(ghz, 3)}


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
    # a step takes about 0.27 ms: a few hundred of them, so that starting and draining the stream (about half a
    # millisecond between the two host clock readings) does not weigh on the figure
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernels", action="store_true", help="skip the separate quantizer / decode timings")
    ap.add_argument("--layout", choices=["matrix", "fragment"], default="matrix",
                    help="operand layout of the prefill product: block-scaled matrix cores (default) or int8 MFMA")
    ap.add_argument("--unfused", action="store_true", help="mx_quantize + mx_pack instead of mx_quantize_pack")
    ap.add_argument("--min-launches", type=int, default=MIN_LAUNCHES,
                    help="launches behind every per-kernel figure (lower it for counter-collection runs)")
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
    # every call of the step marshalled once, every event created before the clock starts: the host then only
    # issues, and the gaps between kernels are the GPU's own
    for w in work:
        c = w["case"]
        if args.unfused:
            w["q_calls"] = [(mx.bound("mx_quantize", x, 1, c.M, c.K, c.K, 0, 1, w["fa"], w["mant"], w["exps"]),
                             mx.bound("mx_pack", w["mant"], w["exps"], 1, c.M, c.K, w["fa"], L, w["A"])) for x in w["xs"]]
        else:
            w["q_calls"] = [(mx.bound("mx_quantize_pack", x, 1, c.M, c.K, c.K, 0, w["fa"], L, w["A"]),) for x in w["xs"]]
        w["g_calls"] = [mx.bound("mx_gemm", 1, c.M, c.N, c.K, w["A"], w["fa"], w["B"], w["fb"], L, y, c.N, 0) for y in w["Y"]]
    hip_events = HipEvents(2 * len(work) * args.steps, torch.cuda.current_stream().cuda_stream)

    def step(i, events):
        for wi, w in enumerate(work):
            for call in w["q_calls"][i % ring]:
                call()
            if events:
                e0 = 2 * (i * len(work) + wi)
                hip_events.record(e0)
            w["g_calls"][i % 2]()
            if events:
                hip_events.record(e0 + 1)
                gemm_events.append((e0, e0 + 1, wi))

    step(0, False)                    # the packed activations of every linear exist before anything reads them
    torch.cuda.synchronize()

    def time_launches(fn, n):
        """Median over batches of the mean time per launch: batches of n back-to-back launches between two
        events, at least MIN_LAUNCHES launches in all (never fewer than 5 batches)."""
        if args.min_launches < MIN_LAUNCHES:          # counter-collection runs: a handful of launches per kernel
            n = max(1, min(n, args.min_launches))
        batches = max(5, -(-args.min_launches // n)) if args.min_launches >= MIN_LAUNCHES else 1
        ms = []
        for _ in range(batches):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(n):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1) / n)
        return float(np.median(ms))

    # what the bare matrix pipe and bare streaming kernels reach on this GPU (the achievable denominators)
    probes = Probes(torch, dev)
    achievable = None
    if not args.no_kernels:
        fp6z, fp6r = probes.mfma("fp6", "zeros"), probes.mfma("fp6", "random")
        i8z, i8r = probes.mfma("i8", "zeros"), probes.mfma("i8", "random")
        big = 1 << 30
        # the product takes two 6-bit instructions per int8-equivalent instruction (8-bit activations = two pieces)
        eq = fp6r["TOPS"] / 2
        achievable = {
            "mfma_fp6_loop_zeros": fp6z, "mfma_fp6_loop_random": fp6r,
            "mfma_i8_loop_zeros": i8z, "mfma_i8_loop_random": i8r,
            "int8_equivalent_TOPS_of_two_piece_fp6_random": round(eq, 1),
            "stream_read_1GiB_GBps": round(big / probes.stream_ms("read", big, time_launches) / 1e6, 1),
            "stream_write_1GiB_GBps": round(big / probes.stream_ms("write", big, time_launches) / 1e6, 1),
            "stream_copy_512MiB_GBps": round(big / probes.stream_ms("copy", big // 2, time_launches) / 1e6, 1)}

    def with_floor(entry, nbytes, ms):
        """Adds the time a bare streaming read of the same number of bytes takes on this GPU, and the kernel's
        time as a fraction of it (a read is the fastest way to touch that many bytes)."""
        floor = probes.stream_ms("read", nbytes, time_launches)
        entry["read_floor_us"] = round(floor * 1e3, 2)
        entry["frac_of_read_floor"] = round(floor / ms, 4)
        return entry

    # ---------------------------------------------------------------- HBM-bound kernels on their own
    kernels = {}
    if not args.no_kernels:
        # the product on its own, back to back on one set of buffers (the operands then stay in the last-level
        # cache between launches, unlike inside a step), and the same on all-zero operands: the instruction
        # stream and its cycle count are the same, but zero operands leave the shader clock where it idles,
        # so the pair tells how much of the product's time is the clock that its operand bits cost
        if args.layout == "matrix":
            for w in work:
                c = w["case"]
                tag = "gemm_%dx%dx%d" % (c.M, c.N, c.K)
                zA, zB = torch.zeros_like(w["A"]), torch.zeros_like(w["B"])
                zero = mx.bound("mx_gemm", 1, c.M, c.N, c.K, zA, w["fa"], zB, w["fb"], L, w["Y"][0], c.N, 0)
                for name, call in (("back_to_back", w["g_calls"][0]), ("zero_operands", zero)):
                    ms = time_launches(lambda i: call(), 25)
                    kernels["%s_%s" % (tag, name)] = {
                        "us": round(ms * 1e3, 2), "TOPS": round(w["ops"] / ms / 1e9, 1),
                        "frac_int8_peak": round(w["ops"] / ms / 1e9 / INT8_MFMA_PEAK_TOPS, 4)}
                del zA, zB
        # quantizer: 4 bytes read + w/8 + 1/block bytes written per element, over a ring of distinct inputs
        # (> 1 GB in all) so that nothing is served from the last-level cache
        for w in (work[0], work[2]):
            c = w["case"]
            nring = int(1.3e9 // (c.M * c.K * 4)) + 1
            qring = [torch.randn((c.M, c.K), dtype=torch.float32, device=dev) for _ in range(nring)]
            # pre-marshalled calls: per-call marshalling in Python would cost as much as these kernels run
            qcalls = [mx.bound("mx_quantize", q, 1, c.M, c.K, c.K, 0, 1, w["fa"], w["mant"], w["exps"]) for q in qring]
            ms = time_launches(lambda i: qcalls[i % nring](), 2 * nring)
            qbytes = c.M * c.K * (4 + c.wx / 8 + 1 / c.block)
            kernels["quantize_%dx%d_w%d_b%d" % (c.M, c.K, c.wx, c.block)] = with_floor({
                "GBps": round(qbytes / ms / 1e6, 1), "frac_hbm": round(qbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                "us": round(ms * 1e3, 2), "bytes": int(qbytes)}, qbytes, ms)
            if c.K == 11008:
                # the paper's own block shape: 16 columns x 2 rows per exponent, MXInt((16,2),8,7)
                f2 = mx.fmt(16, 8, block_rows=2)
                e2 = torch.empty(mx.mx_exps_bytes(1, c.M, c.K, f2), dtype=torch.uint8, device=dev)
                qcalls = [mx.bound("mx_quantize", q, 1, c.M, c.K, c.K, 0, 1, f2, w["mant"], e2) for q in qring]
                ms = time_launches(lambda i: qcalls[i % nring](), 2 * nring)
                kernels["quantize_%dx%d_w8_b16x2" % (c.M, c.K)] = with_floor({
                    "GBps": round(qbytes / ms / 1e6, 1), "frac_hbm": round(qbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                    "us": round(ms * 1e3, 2), "bytes": int(qbytes)}, qbytes, ms)
            if c.K == 11008:
                # the paper's other block formats at the same shape: Block Minifloat (1 + 4 + 3 bits) and Block
                # Logarithm (1 + 7 bits), one byte per element + one shared byte per block
                mcodes = torch.empty(c.M * c.K, dtype=torch.uint8, device=dev)
                mshared = torch.empty(c.M * c.K // c.block, dtype=torch.uint8, device=dev)
                for name, fm in (("bmf_e4m3", mx.mx_minifloat_format(c.block, 4, 3, mx.MX_RNE)),
                                 ("bl_e7", mx.mx_minifloat_format(c.block, 7, 0, mx.MX_RNE))):
                    qcalls = [mx.bound("mx_quantize_minifloat", q, 1, c.M, c.K, c.K, 0, fm, mcodes, mshared) for q in qring]
                    ms = time_launches(lambda i: qcalls[i % nring](), 2 * nring)
                    mbytes = c.M * c.K * (4 + 1 + 1 / c.block)
                    kernels["quantize_%s_%dx%d_b%d" % (name, c.M, c.K, c.block)] = with_floor({
                        "GBps": round(mbytes / ms / 1e6, 1), "frac_hbm": round(mbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                        "us": round(ms * 1e3, 2), "bytes": int(mbytes)}, mbytes, ms)
            if args.layout == "matrix":
                qcalls = [mx.bound("mx_quantize_pack", q, 1, c.M, c.K, c.K, 0, w["fa"], L, w["A"]) for q in qring]
                ms = time_launches(lambda i: qcalls[i % nring](), 2 * nring)
                pbytes = c.M * c.K * 4 + mx.mx_packed_bytes(1, c.M, c.K, w["fa"], L)
                kernels["quantize_pack_matrix_%dx%d_w%d_b%d" % (c.M, c.K, c.wx, c.block)] = with_floor({
                    "GBps": round(pbytes / ms / 1e6, 1), "frac_hbm": round(pbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                    "us": round(ms * 1e3, 2), "bytes": int(pbytes)}, pbytes, ms)
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
        kernels["cast_%dx%d_w8_to_w4_b%d" % (c.M, c.K, c.block)] = with_floor({
            "GBps": round(cbytes / ms / 1e6, 1), "frac_hbm": round(cbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
            "us": round(ms * 1e3, 2), "bytes": int(cbytes)}, cbytes, ms)
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
                kernels["linear_%s_M%d" % (dc.name, M)] = with_floor({
                    "GBps": round(nbytes / ms / 1e6, 1), "frac_hbm": round(nbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                    "us": round(ms * 1e3, 2), "bytes": int(nbytes)}, nbytes, ms)
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
            e = with_floor({"GBps": round(nbytes / ms / 1e6, 1), "frac_hbm": round(nbytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                            "us": round(ms * 1e3, 2), "bytes": int(nbytes)}, nbytes, ms)
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

    # ---------------------------------------------------------------- the steps
    # They come after the sections above on purpose: with the driver's five warm-up steps on a GPU that has just been
    # set up, the first few dozen steps run 10 - 15 % slower than the ones after them (20 timed steps: 0.29 - 0.31 ms
    # per step after 5 warm-up steps, 0.26 after 50, 0.25 after 400, with the product's own launches slower as well);
    # behind a second of kernel timings the GPU is in the state it keeps under sustained work.
    def timed_steps():
        if args.calibrate_copy:
            src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
            dst = torch.empty_like(src)
            dst.copy_(src)
            torch.cuda.synchronize()
            del src, dst
        for i in range(args.warmup):
            step(i, False)
        # the timed region: K steps, nothing but the library's launches on the stream
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i, False)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        sec = t1 - t0
        ms_per_step = 1e3 * sec / args.steps
        value = total_ops * args.steps / sec / 1e12

        # the same K steps again with a HIP event on either side of every mx_gemm: the product's launch durations
        # inside the step (each event costs the stream a few microseconds, which is why the region above has none)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i, True)
        torch.cuda.synchronize()
        ms_per_step_events = 1e3 * (time.perf_counter() - t0) / args.steps

        per_shape = []
        for wi, w in enumerate(work):
            ms = [hip_events.elapsed_ms(e0, e1) for e0, e1, k in gemm_events if k == wi]
            c = w["case"]
            per_shape.append({"shape": "%dx%dx%d" % (c.M, c.N, c.K), "launches": len(ms),
                              "avg_launch_us": round(1e3 * sum(ms) / len(ms), 2),
                              "TOPS": round(w["ops"] / (sum(ms) / len(ms) * 1e-3) / 1e12, 1)})
        gemm_ms = sum(hip_events.elapsed_ms(e0, e1) for e0, e1, _ in gemm_events)
        hip_events.destroy()
        gemm_ops = sum(work[k]["ops"] for _, _, k in gemm_events)
        achieved = gemm_ops / (gemm_ms * 1e-3) / 1e12
        kname = ("mx_gemm (block-scaled fp6 MFMA, two mantissa pieces for 8-bit activations)" if args.layout == "matrix"
                 else "mx_gemm (int8 MFMA, block-exponent epilogue)")
        roofline = {"kernel": kname, "bound": "mfma",
                    "achieved": round(achieved, 2), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                    "frac": round(achieved / INT8_MFMA_PEAK_TOPS, 4),
                    "traffic": recorded_traffic() if args.layout == "matrix" else None,
                    "avg_launch_ms": round(gemm_ms / len(gemm_events), 4),
                    "per_shape": per_shape,
                    "ms_per_step_with_events": round(ms_per_step_events, 4)}
        return value, ms_per_step, roofline

    value, ms_per_step, roofline = timed_steps()
    if achievable is not None:
        eq = achievable["int8_equivalent_TOPS_of_two_piece_fp6_random"]
        achievable["frac_of_achievable"] = round(roofline["achieved"] / eq, 4)
        roofline["achievable"] = achievable

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
