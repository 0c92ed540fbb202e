#!/usr/bin/env python3
"""Benchmark of the w2a8 hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch: for each of the
four projections of an 8B-class decoder layer (QKV, O, gate+up, down) at M=1,
quantise the fp32 activation row to int8 (per token) and run the 2-bit-weight
matmul with its fused dequant (bf16 out).  By default quantisation runs inside
the matmul kernel (w2_matmul_a8_fused: one launch per projection, the paper's
fused GPU design, bit-identical to the two-call path); the two-call path
(w2_quantize_rows + w2_matmul_a8) is timed beside it.  Weights are prepacked once (off-line step)
and resident in HBM; successive steps walk a pool of distinct prepacked layers
larger than twice the 256 MB last-level cache, so every step streams its
weights from HBM as a real decode does.  Steps are replayed from HIP graphs, one
graph per pass over the pool (13 consecutive steps, as a decode loop captures a
whole token's pass over its layers), so that host launch cost does not hide the
GPU time: with one graph per step the host's graph launches set the pace
(28.4 against 23.7 us per step).

Prints ONE JSON line: metric / value / unit (whole-step GB/s of the method's own bytes), the
`roofline` of the dominant kernel, `prefill` (compute-bound TOP/s), `cpu_baseline` (the oracle).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
INT8_PEAK_TOPS = 5000.0        # dense int8 MFMA peak
POOL_BYTES = 704 << 20         # > 2 x 256 MB last-level cache
G = 128


def algorithmic_bytes(M, K, N, g=G):
    """Bytes the method itself must move for one matmul call: 2-bit codes, group
    scales, int8 activations in, bf16 out."""
    return K * N // 4 + (K // g) * N * 2 + M * K + 2 * M * N


def read_traffic(kernel_key):
    """HBM bytes per launch of a kernel as measured with `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE`
    (two runs of `bench.py --pmc`, scaled by the plain copy); the summary under profiles/ carries a
    line `traffic_bytes_per_launch[<key>] = <bytes>`.  None when no such measurement is on file."""
    path = os.path.join(ROOT, "profiles", "pmc_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch[%s]" % kernel_key):
                return int(float(line.rsplit("=", 1)[1].split()[0]))
    except OSError:
        pass
    return None


def pmc_mode(torch, w2, lib, vp, pool, shapes, Xd, Yd, dev):
    import ctypes
    M = 1
    s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    src = torch.randint(0, 255, (256 << 20,), dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    Kd, Nd = shapes["gate_up"]
    for _ in range(3):
        dst.copy_(src)                                   # calibration: reads 256 MiB, writes 256 MiB
    for l in pool:
        lib.w2_debug_stream_read(vp(l["gate_up"]), l["gate_up"].numel(), vp(sink), None, s)
    for name in ("gate_up", "down", "qkv", "o"):             # the step's four fused launches, one projection at a time
        Kq, Nq = shapes[name]
        for l in pool:
            rc = lib.w2_matmul_a8_fused(vp(l[name]), Kq, Nq, G, vp(Xd[name]), w2.DT_F32, Kq, M,
                                        vp(Yd[name]), Nq, None, 0, s)
            assert rc == 0, lib.w2_last_error()
    Kp, Np, Mp = 8192, 57344, 2048
    pk = torch.randint(0, 255, (w2.packed_size(Kp, Np, G),), dtype=torch.uint8, device=dev)
    pk[Kp * Np // 4:].view(torch.int16)[:] = 0x3C00
    xqp = torch.randint(-127, 128, (Mp, Kp), dtype=torch.int8, device=dev)
    sxp = torch.rand(Mp, device=dev)
    Yp = torch.empty((Mp, Np), dtype=torch.bfloat16, device=dev)
    for _ in range(3):
        w2.matmul_a8(pk, Kp, Np, G, xqp, sxp, out=Yp)
    xbp = torch.randn((Mp, Kp), dtype=torch.bfloat16, device=dev)
    for _ in range(3):
        w2.matmul_a16(pk, Kp, Np, G, xbp, out=Yp)
    torch.cuda.synchronize()
    print("bench.py --pmc: launched copy x3 (256 MiB), stream read x%d, fused GEMV x%d on gate+up, down, QKV, O, "
          "prefill x3 (w2a8), x3 (w2a16)" % (len(pool), len(pool)))


def probe_sweep_mode(torch, w2, synth, dev):
    """Launch-shape sweep of the streaming-read probe (the ceiling the decode kernels are compared with) on the
    four 8B-class blobs: chunks in flight per wave x most workgroups, graph-timed over a pool of copies."""
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    for name, (K, N) in synth.SHAPES_8B.items():
        nb = w2.packed_size(K, N, G)
        n = max(2, -(-POOL_BYTES // nb))
        base = torch.randint(0, 255, (nb,), dtype=torch.uint8, device=dev)
        pool = [base] + [base.clone() for _ in range(n - 1)]
        for u in (4, 8, 16):
            for b in (256, 512, 1024, 2048, 4096, 8192, 16384):
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr):
                    for l in pool:
                        w2.debug_stream_read(l, sink, tune={"stream_unroll": u, "stream_blocks": b})
                t_end = time.perf_counter() + 0.05
                while time.perf_counter() < t_end:
                    gr.replay()
                    torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(6):
                    gr.replay()
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / (6 * len(pool))
                print("probe %-8s %9d B unroll=%2d blocks=%5d %7.2f us %7.1f GB/s" % (name, nb, u, b, us, nb / us / 1e3), flush=True)
        del pool


def gamma_mode(torch, w2, synth, dev, timing):
    """The small-batch sweep (gate+up 4096 x 28672, M in {1,2,4,8,16}, G in {64,128}) through every w2a8 kernel
    family that covers the M.  With `timing` each case is graph-timed over a pool of weight copies (one line
    per case); without it each case is launched eagerly three times, in the same order, for `rocprofv3 --pmc`
    to count its instructions (the line then carries the case's position in the dispatch order)."""
    K, N = synth.SHAPES_8B["gate_up"]
    fam = [("gemv", w2.VARIANT_GEMV, 16), ("dot4", w2.VARIANT_DOT4, 4), ("smallm", w2.VARIANT_SMALLM, 16),
           ("midm", w2.VARIANT_MIDM, 64)]
    pos = 0
    for g in (128, 64):
        nb = w2.packed_size(K, N, g)
        n = max(2, -(-POOL_BYTES // nb)) if timing else 1
        base = torch.randint(0, 255, (nb,), dtype=torch.uint8, device=dev)
        base[K * N // 4:].view(torch.int16)[:] = 0x3C00
        pool = [base] + [base.clone() for _ in range(n - 1)]
        for M in (1, 2, 4, 8, 16):
            X = torch.randn(M, K, device=dev)
            xq, sx, _ = w2.quantize_rows(X, g)
            Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
            pos += 1                                          # the quantise launch
            for name, variant, m_max in fam:
                if M > m_max:
                    continue
                words = K * N // 16                           # 32-bit code words per launch
                if timing:
                    gr = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(gr):
                        for l in pool:
                            w2.matmul_a8(l, K, N, g, xq, sx, out=Y, variant=variant)
                    t_end = time.perf_counter() + 0.1
                    while time.perf_counter() < t_end:
                        gr.replay()
                        torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(6):
                        gr.replay()
                    e1.record()
                    torch.cuda.synchronize()
                    us = e0.elapsed_time(e1) * 1e3 / (6 * len(pool))
                    by = algorithmic_bytes(M, K, N, g)
                    print("gamma G=%3d M=%2d %-6s %8.2f us %8.1f GB/s  code words %d" % (g, M, name, us, by / us / 1e3, words),
                          flush=True)
                else:
                    for _ in range(3):
                        w2.matmul_a8(pool[0], K, N, g, xq, sx, out=Y, variant=variant)
                    print("gamma G=%3d M=%2d %-6s dispatches %d..%d  code words %d" % (g, M, name, pos, pos + 2, words), flush=True)
                    pos += 3
    torch.cuda.synchronize()


def sweep_mode(torch, w2, synth, dev, sections=None):
    """One line per (configuration, projection, M, call): microseconds per launch, the method's own
    bytes / time (GB/s, % of 8 TB/s) for M <= 64, ops / time (TOP/s, % of the MFMA peak) above."""
    def pool_for(K, N, g):
        nb = w2.packed_size(K, N, g)
        n = max(2, -(-POOL_BYTES // nb))
        base = torch.randint(0, 255, (nb,), dtype=torch.uint8, device=dev)      # any bytes are valid codes
        base[K * N // 4:].view(torch.int16)[:] = 0x3C00                         # scales region: finite bf16
        return [base] + [base.clone() for _ in range(n - 1)]

    def timed(fn, pool, reps=6):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for l in pool:
                fn(l)
        t_end = time.perf_counter() + 0.1
        while time.perf_counter() < t_end:
            g.replay()
            torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * len(pool))

    def line(cfg, name, K, N, g, M, call, us):
        if M <= 64:
            act = {"a8": M * K, "a8 fused(f32 in)": 4 * M * K, "a16": 2 * M * K, "stream read": 0}[call]
            by = K * N // 4 + (K // g) * N * 2 + act + (0 if call == "stream read" else 2 * M * N)
            rate = "%8.1f GB/s %5.1f%% of 8 TB/s" % (by / us / 1e3, by / us / 1e3 / HBM_PEAK_GBS * 100)
        else:
            tops = 2.0 * M * K * N / us / 1e6
            peak = 2500.0 if call == "a16" else INT8_PEAK_TOPS
            rate = "%8.1f TOP/s %5.1f%% of %.1f POP/s" % (tops, tops / peak * 100, peak / 1e3)
        print("%-6s %-8s K=%5d N=%5d G=%3d M=%4d %-17s %9.2f us  %s" % (cfg, name, K, N, g, M, call, us, rate), flush=True)

    def decode_case(cfg, name, K, N, g, Ms, calls):
        if sections and cfg not in sections:
            return
        pool = pool_for(K, N, g)
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        if "stream read" in calls:
            line(cfg, name, K, N, g, 1, "stream read", timed(lambda l: w2.debug_stream_read(l, sink), pool))
        for M in Ms:
            X = torch.randn(M, K, device=dev)
            xq, sx, _ = w2.quantize_rows(X, g)
            Xb = X.to(torch.bfloat16)
            Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
            nws = w2.workspace_size(M, K, N, g)
            ws = torch.empty(nws, dtype=torch.uint8, device=dev) if nws else None
            nws16 = w2.workspace_size(M, K, N, g, a16=True)
            ws16 = torch.empty(nws16, dtype=torch.uint8, device=dev) if nws16 else None
            if "a8" in calls:
                line(cfg, name, K, N, g, M, "a8", timed(lambda l: w2.matmul_a8(l, K, N, g, xq, sx, out=Y, workspace=ws), pool))
            if "fused" in calls:
                line(cfg, name, K, N, g, M, "a8 fused(f32 in)",
                     timed(lambda l: w2.matmul_a8_fused(l, K, N, g, X, out=Y, workspace=ws), pool))
            if "a16" in calls:
                line(cfg, name, K, N, g, M, "a16",
                     timed(lambda l: w2.matmul_a16(l, K, N, g, Xb, out=Y, workspace=ws16), pool))
        del pool

    print("# every launch reads a different prepacked copy (pool > 2 x 256 MB last-level cache); times are per launch "
          "inside a replayed HIP graph, gaps between launches included")
    decode_case("cfg0", "single", 2048, 2048, 128, (1,), ("a8", "fused", "stream read"))
    for name, (K, N) in synth.SHAPES_8B.items():
        decode_case("cfg1", name, K, N, 128, (1, 4, 8), ("a8", "fused", "a16", "stream read"))
    for g in (128, 64):
        decode_case("cfg2", "gate_up", 4096, 28672, g, (1, 2, 4, 8, 16, 32, 64), ("a8",))
    for name, (K, N) in synth.SHAPES_27B.items():
        decode_case("cfg3", name, K, N, 128, (1, 8), ("a8", "fused", "stream read"))
    print("# between decode and prefill (8B-class projections; workspaces of w2_workspace_size bytes, so the tiled "
          "kernels may split K)")
    for name, (K, N) in synth.SHAPES_8B.items():
        decode_case("mid", name, K, N, 128, (16, 32, 64, 128, 256), ("a8", "a16"))
    print("# the same between decode and prefill on the deepest projection (70B-class down, 28672 x 8192)")
    decode_case("deep", "down", 28672, 8192, 128, (16, 32, 64, 128, 256), ("a8", "a16"))
    if sections and "cfg4" not in sections:
        return
    print("# prefill: 40 launches and 0.15 s to warm the clock up, 20 timed; workspaces of w2_workspace_size bytes (none needed at M = 2048)")
    for name, (K, N) in synth.SHAPES_70B.items():
        nb = w2.packed_size(K, N, G)
        pk = torch.randint(0, 255, (nb,), dtype=torch.uint8, device=dev)
        pk[K * N // 4:].view(torch.int16)[:] = 0x3C00
        for M in (512, 2048):
            X = torch.randn(M, K, device=dev)
            xq, sx, _ = w2.quantize_rows(X, G)
            Xb = X.to(torch.bfloat16)
            del X
            Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
            nws, nws16 = w2.workspace_size(M, K, N, G), w2.workspace_size(M, K, N, G, a16=True)
            ws = torch.empty(nws, dtype=torch.uint8, device=dev) if nws else None
            ws16 = torch.empty(nws16, dtype=torch.uint8, device=dev) if nws16 else None
            for call, fn in (("a8", lambda: w2.matmul_a8(pk, K, N, G, xq, sx, out=Y, workspace=ws)),
                             ("a16", lambda: w2.matmul_a16(pk, K, N, G, Xb, out=Y, workspace=ws16))):
                for _ in range(40 if call == "a8" else 15):
                    fn()
                torch.cuda.synchronize()
                t_end = time.perf_counter() + 0.15            # ... and until the chip has been busy for a while: the
                while time.perf_counter() < t_end:           # first case of a cold chip otherwise reads 10 % slow
                    fn()
                    torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                n = 20 if call == "a8" else 8
                e0.record()
                for _ in range(n):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                line("cfg4", name, K, N, G, M, call, e0.elapsed_time(e1) * 1e3 / n)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--pmc", action="store_true",
                    help="counter-collection mode for `rocprofv3 --pmc`: launch, eagerly and a few times each, a plain "
                         "256 MiB device copy (the calibration kernel), the streaming read, the dominant GEMV over "
                         "the pool and the prefill kernel; print no bench line")
    ap.add_argument("--probe-sweep", action="store_true",
                    help="launch-shape sweep of the streaming-read probe on the 8B-class blobs (a table, no bench line)")
    ap.add_argument("--gamma", choices=["time", "count"],
                    help="the small-batch sweep on gate+up (M = 1..16, G = 64 and 128, every w2a8 kernel family): "
                         "`time` prints graph-timed microseconds per launch, `count` launches each case eagerly "
                         "three times for `rocprofv3 --pmc` (vector instructions per 32-bit code word)")
    ap.add_argument("--sweep", action="store_true",
                    help="time every configuration BASELINE.json lists (decode shapes from HIP graphs over a pool "
                         "of distinct weight copies, prefill shapes under sustained launches) and print a table "
                         "instead of the bench line")
    ap.add_argument("--sections", default="",
                    help="with --sweep: only these sections of the table (comma-separated: cfg0..cfg4, mid, deep)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); "
                 "use --gpus 1.")

    import numpy as np
    import torch
    from paper_2508_06753_amd import binding as w2, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    if args.sweep:
        return sweep_mode(torch, w2, synth, dev, set(args.sections.split(",")) - {""} or None)
    if args.probe_sweep:
        return probe_sweep_mode(torch, w2, synth, dev)
    if args.gamma:
        return gamma_mode(torch, w2, synth, dev, args.gamma == "time")
    M = 1
    shapes = synth.SHAPES_8B

    def to_dev(a):
        if a.dtype == np.uint16:
            a = a.view(np.int16)
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    # ---- synthetic layer (seed 1), prepacked once; the pool holds copies of the packed blobs
    # (kernel time does not depend on the values, only on the bytes streamed)
    host = {}
    packed0 = {}
    for i, (name, (K, N)) in enumerate(shapes.items()):
        codes, scales, X = synth.make_problem(M, K, N, G, synth.CODEC_INT2, seed=1 + i)
        host[name] = (codes, scales, X)
        packed0[name] = w2.prepack(to_dev(codes), to_dev(scales), G, w2.CODEC_INT2)
    layer_bytes = sum(p.numel() for p in packed0.values())
    n_pool = max(2, -(-POOL_BYTES // layer_bytes))
    pool = [packed0] + [{k: v.clone() for k, v in packed0.items()} for _ in range(n_pool - 1)]
    Xd = {name: to_dev(host[name][2]) for name in shapes}
    Yd = {name: torch.empty((M, shapes[name][1]), dtype=torch.bfloat16, device=dev) for name in shapes}
    xq = {name: torch.empty((M, shapes[name][0]), dtype=torch.int8, device=dev) for name in shapes}
    sx = {name: torch.empty((M,), dtype=torch.float32, device=dev) for name in shapes}

    import ctypes
    lib = w2.raw()

    def vp(t):
        return ctypes.c_void_p(t.data_ptr())

    def step(layer):
        s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        for name, (K, N) in shapes.items():
            rc = lib.w2_matmul_a8_fused(vp(layer[name]), K, N, G, vp(Xd[name]), w2.DT_F32, K, M,
                                        vp(Yd[name]), N, None, 0, s)
            assert rc == 0, lib.w2_last_error()

    def step_two_call(layer):
        s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        for name, (K, N) in shapes.items():
            rc = lib.w2_quantize_rows(vp(Xd[name]), w2.DT_F32, M, K, K, G, vp(xq[name]), vp(sx[name]),
                                      None, s)
            assert rc == 0, lib.w2_last_error()
            rc = lib.w2_matmul_a8(vp(layer[name]), K, N, G, vp(xq[name]), vp(sx[name]), M,
                                  vp(Yd[name]), N, None, 0, s)
            assert rc == 0, lib.w2_last_error()

    def capture(fn):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g

    step(pool[0])
    step_two_call(pool[0])
    torch.cuda.synchronize()
    if args.pmc:
        return pmc_mode(torch, w2, lib, vp, pool, shapes, Xd, Yd, dev)
    use_graph = os.environ.get("W2_BENCH_NO_GRAPH", "0") != "1"

    class Steps:
        """Runs exactly n steps of `fn`, step i on pool layer i % n_pool.  With graphs: one HIP graph holds
        n_pool consecutive steps (a decode loop captures a whole token's pass over the layers, not one layer
        per graph: with a graph per step the host's graph launch, not the GPU, sets the pace), and one more
        graph holds the n % n_pool steps left over."""

        def __init__(self, fn):
            self.fn = fn
            self.graphs = {}

        def graph(self, n):
            if n not in self.graphs:
                self.graphs[n] = capture(lambda: [self.fn(pool[i]) for i in range(n)])
            return self.graphs[n]

        def prepare(self, *counts):
            if use_graph:
                for n in counts:
                    self.graph(n_pool)
                    if n % n_pool:
                        self.graph(n % n_pool)

        def run(self, n):
            if not use_graph:
                for i in range(n):
                    self.fn(pool[i % n_pool])
                return
            for _ in range(n // n_pool):
                self.graphs[n_pool].replay()
            if n % n_pool:
                self.graphs[n % n_pool].replay()

    fused_steps, two_call_steps = Steps(step), Steps(step_two_call)
    fused_steps.prepare(args.steps, args.warmup)
    two_call_steps.prepare(args.steps, args.warmup)

    # the chip raises its clocks only under sustained load: keep it busy for a quarter of a second
    # before the counted warm-up, so that timed steps do not run on the ramp
    t_end = time.perf_counter() + 0.25
    while time.perf_counter() < t_end:
        fused_steps.run(4 * n_pool)
        torch.cuda.synchronize()
    fused_steps.run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    fused_steps.run(args.steps)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = wall_ms / args.steps
    gpu_ms_per_step = e0.elapsed_time(e1) / args.steps
    step_bytes = sum(algorithmic_bytes(M, K, N) for K, N in shapes.values())
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # the same step with separate quantise launches, for comparison
    two_call_steps.run(args.warmup)
    torch.cuda.synchronize()
    e0.record()
    two_call_steps.run(args.steps)
    e1.record()
    torch.cuda.synchronize()
    two_call_ms = e0.elapsed_time(e1) / args.steps

    # ---- the same layer as a dependent chain, one graph per pool entry: QKV -> (attention left out: the
    # first 4096 outputs stand in for its result) -> O -> gate+up with the gated SiLU epilogue -> down.
    # Every call takes the previous call's bf16 output and quantises it inside the kernel.
    Kq, Nq = shapes["qkv"]
    Ko, No = shapes["o"]
    Kg, Ng = shapes["gate_up"]
    Kdn, Ndn = shapes["down"]
    assert Ko <= Nq and Kg == No and Kdn == Ng // 2
    c_qkv = torch.empty((1, Nq), dtype=torch.bfloat16, device=dev)
    c_o = torch.empty((1, No), dtype=torch.bfloat16, device=dev)
    c_act = torch.empty((1, Ng // 2), dtype=torch.bfloat16, device=dev)
    c_out = torch.empty((1, Ndn), dtype=torch.bfloat16, device=dev)

    def step_chained(layer):
        s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        rc = lib.w2_matmul_a8_fused(vp(layer["qkv"]), Kq, Nq, G, vp(Xd["qkv"]), w2.DT_F32, Kq, M, vp(c_qkv), Nq, None, 0, s)
        assert rc == 0, lib.w2_last_error()
        rc = lib.w2_matmul_a8_fused(vp(layer["o"]), Ko, No, G, vp(c_qkv), w2.DT_BF16, Nq, M, vp(c_o), No, None, 0, s)
        assert rc == 0, lib.w2_last_error()
        w2.matmul_a8_fused_epi(layer["gate_up"], Kg, Ng, G, c_o, act=w2.ACT_SILU_MUL, out=c_act)
        rc = lib.w2_matmul_a8_fused(vp(layer["down"]), Kdn, Ndn, G, vp(c_act), w2.DT_BF16, Kdn, M, vp(c_out), Ndn, None, 0, s)
        assert rc == 0, lib.w2_last_error()

    step_chained(pool[0])
    torch.cuda.synchronize()
    chained_steps = Steps(step_chained)
    chained_steps.prepare(args.steps, args.warmup)
    chained_steps.run(args.warmup)
    torch.cuda.synchronize()
    e0.record()
    chained_steps.run(args.steps)
    e1.record()
    torch.cuda.synchronize()
    chained_ms = e0.elapsed_time(e1) / args.steps
    chained_bytes = step_bytes - 2 * M * (Ng // 2)           # the gated epilogue stores half the columns

    # ---- roofline of the dominant kernel: the GEMV on the largest projection (gate+up),
    # launched alone, back to back over the pool, timed with events on the launch stream
    Kd, Nd = shapes["gate_up"]

    def gemv_only(layer):
        s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        rc = lib.w2_matmul_a8_fused(vp(layer["gate_up"]), Kd, Nd, G, vp(Xd["gate_up"]), w2.DT_F32, Kd, M,
                                    vp(Yd["gate_up"]), Nd, None, 0, s)
        assert rc == 0, lib.w2_last_error()

    def all_gemv():
        for l in pool:
            gemv_only(l)

    gg = capture(all_gemv) if use_graph else None
    reps = 20
    for _ in range(3):
        gg.replay() if gg else all_gemv()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        gg.replay() if gg else all_gemv()
    e1.record()
    torch.cuda.synchronize()
    gemv_us = e0.elapsed_time(e1) * 1e3 / (reps * n_pool)
    gemv_bytes = algorithmic_bytes(M, Kd, Nd)
    achieved = gemv_bytes / gemv_us / 1e3           # GB/s

    # attainable read ceiling: a plain 128-bit streaming read of the same number of bytes
    sink = torch.zeros(1, dtype=torch.int32, device=dev)

    def all_read():
        s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        for l in pool:
            lib.w2_debug_stream_read(vp(l["gate_up"]), l["gate_up"].numel(), vp(sink), None, s)

    gr = capture(all_read) if use_graph else None
    for _ in range(3):
        gr.replay() if gr else all_read()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        gr.replay() if gr else all_read()
    e1.record()
    torch.cuda.synchronize()
    read_us = e0.elapsed_time(e1) * 1e3 / (reps * n_pool)

    # the paper's own comparator: an int8-weight GEMV of the same shape (four times the bytes, no
    # up-convert), over a pool of distinct copies as well
    n8 = max(2, -(-POOL_BYTES // (Kd * Nd)))
    W8 = torch.randint(-128, 128, (Nd, Kd), dtype=torch.int8, device=dev)
    pool8 = [W8] + [W8.clone() for _ in range(n8 - 1)]
    xq8 = torch.randint(-127, 128, (Kd,), dtype=torch.int8, device=dev)
    out8 = torch.empty(Nd, dtype=torch.int32, device=dev)

    def all_int8():
        for w in pool8:
            w2.debug_int8_gemv(w, xq8, out=out8)

    g8 = capture(all_int8) if use_graph else None
    for _ in range(3):
        g8.replay() if g8 else all_int8()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        g8.replay() if g8 else all_int8()
    e1.record()
    torch.cuda.synchronize()
    int8_us = e0.elapsed_time(e1) * 1e3 / (reps * n8)
    int8_gbs = (Kd * Nd + Kd + 4 * Nd) / int8_us / 1e3
    del pool8, W8

    out = {
        "metric": "M=1 weight-stream GB/s (% of HBM peak); TOPS at M=2048 (% of int8 MFMA peak)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "gpu_ms_per_step": round(gpu_ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": "8B-class decode layer, M=1, w2a8, G=128: quantise + matmul (one fused launch each) for "
                               "QKV 4096x6144, O 4096x4096, gate+up 4096x28672, down 14336x4096",
                   "bytes_per_step": step_bytes, "pool_layers": n_pool, "hip_graph": use_graph,
                   "steps_per_graph": n_pool if use_graph else None,
                   "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
                   "two_call_gpu_ms_per_step": round(two_call_ms, 5),
                   "chained_layer": {"what": "QKV -> O -> gate+up with fused silu(gate)*up -> down, each call fed by the "
                                             "previous call's bf16 output (attention, norms and residuals left out)",
                                     "gpu_ms_per_step": round(chained_ms, 5),
                                     "GBps": round(chained_bytes / (chained_ms * 1e-3) / 1e9, 1)}},
        "roofline": {"bound": "hbm", "kernel": "a8_gemv_kernel, fp32 row in (quantise + int8 MFMA GEMV + dequant) on gate+up 4096x28672, M=1",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": read_traffic("a8_gemv gate_up M=1"),
                     "us_per_launch": round(gemv_us, 3), "bytes_per_launch": gemv_bytes,
                     "stream_read_us_same_bytes": round(read_us, 3),
                     "frac_of_stream_read": round(read_us / gemv_us, 4),
                     "int8_weight_gemv_same_shape": {"us_per_launch": round(int8_us, 3), "GBps": round(int8_gbs, 1),
                                                     "speedup_of_2bit": round(int8_us / gemv_us, 3)}},
    }

    # ---- secondary headline: compute-bound prefill, 70B-class gate+up at M=2048
    if not args.no_prefill:
        Kp, Np, Mp = 8192, 57344, 2048
        nb = w2.packed_size(Kp, Np, G)
        pk = torch.randint(0, 255, (nb,), dtype=torch.uint8, device=dev)   # any bytes are valid weights
        pk[Kp * Np // 4:].view(torch.int16)[:] = 0x3C00                    # scales region: finite bf16
        xqp = torch.randint(-127, 128, (Mp, Kp), dtype=torch.int8, device=dev)
        sxp = torch.rand(Mp, device=dev)
        Yp = torch.empty((Mp, Np), dtype=torch.bfloat16, device=dev)
        # the chip raises its clock only under sustained load: the first few tens of milliseconds
        # of a burst of launches run slower, so warm up for about as long before timing
        for _ in range(40):
            w2.matmul_a8(pk, Kp, Np, G, xqp, sxp, out=Yp)
        torch.cuda.synchronize()
        e0.record()
        nrep = 20
        for _ in range(nrep):
            w2.matmul_a8(pk, Kp, Np, G, xqp, sxp, out=Yp)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / nrep
        tops = 2.0 * Mp * Kp * Np / us / 1e6
        out["prefill"] = {"workload": "70B-class gate+up 8192x57344, M=2048, w2a8, G=128 (matmul only)",
                          "us_per_launch": round(us, 1), "value": round(tops, 1), "unit": "TOPS",
                          "roofline": {"bound": "mfma", "achieved": round(tops, 1), "peak": INT8_PEAK_TOPS,
                                       "unit": "TOP/s", "frac": round(tops / INT8_PEAK_TOPS, 4),
                                       "traffic": read_traffic("a8_tiled gate_up 70B M=2048")}}
        # comparator, as in the paper's GEMM figure: the vendor library's plain int8 x int8 -> int32
        # GEMM (no up-convert, no scales, no bf16 output) on the same shape, weights drawn from the
        # values the 2-bit codes up-convert to, K-contiguous (its faster layout)
        try:
            B8 = (torch.randint(-2, 2, (Np, Kp), dtype=torch.int8, device=dev) * 64).t()
            for _ in range(40):
                torch._int_mm(xqp, B8)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(nrep):
                torch._int_mm(xqp, B8)
            e1.record()
            torch.cuda.synchronize()
            lib_us = e0.elapsed_time(e1) * 1e3 / nrep
            out["prefill"]["library_int8_gemm"] = {"what": "torch._int_mm (hipBLASLt), int8 x int8 -> int32, same shape",
                                                   "us_per_launch": round(lib_us, 1),
                                                   "TOPS": round(2.0 * Mp * Kp * Np / lib_us / 1e6, 1),
                                                   "w2a8_over_library": round(lib_us / us, 3)}
            del B8
        except Exception as e:                               # the comparator is optional
            out["prefill"]["library_int8_gemm"] = {"error": str(e)[:120]}
        # the unquantised-activation variant (w2a16) on the same shape, bf16 MFMA
        Xb = torch.randn(Mp, Kp, device=dev).to(torch.bfloat16)
        for _ in range(25):
            w2.matmul_a16(pk, Kp, Np, G, Xb, out=Yp)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(8):
            w2.matmul_a16(pk, Kp, Np, G, Xb, out=Yp)
        e1.record()
        torch.cuda.synchronize()
        us16 = e0.elapsed_time(e1) * 1e3 / 8
        tf16 = 2.0 * Mp * Kp * Np / us16 / 1e6
        out["prefill_a16"] = {"workload": "the same shape, w2a16 (bf16 activations, bf16 MFMA)", "us_per_launch": round(us16, 1),
                              "value": round(tf16, 1), "unit": "TFLOP/s",
                              "roofline": {"bound": "mfma", "achieved": round(tf16, 1), "peak": 2500.0, "unit": "TFLOP/s",
                                           "frac": round(tf16 / 2500.0, 4),
                                           "traffic": read_traffic("a16_fold_tiled gate_up 70B M=2048")}}
        try:
            B16 = torch.randn(Np, Kp, device=dev, dtype=torch.bfloat16).t()
            for _ in range(15):
                torch.matmul(Xb, B16, out=Yp)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(8):
                torch.matmul(Xb, B16, out=Yp)
            e1.record()
            torch.cuda.synchronize()
            lib16_us = e0.elapsed_time(e1) * 1e3 / 8
            out["prefill_a16"]["library_bf16_gemm"] = {"what": "torch.matmul (hipBLASLt), bf16 x bf16 -> bf16, same shape, 16-bit weights",
                                                       "us_per_launch": round(lib16_us, 1),
                                                       "TFLOPS": round(2.0 * Mp * Kp * Np / lib16_us / 1e6, 1),
                                                       "w2a16_over_library": round(lib16_us / us16, 3)}
            del B16
        except Exception as e:
            out["prefill_a16"]["library_bf16_gemm"] = {"error": str(e)[:120]}
        del pk, xqp, Yp, Xb

    # ---- between the two regimes: the weight stream read once for M = 32 rows (mid-M kernel),
    # and the w2a16 GEMV, both on the 8B gate+up projection over the pool
    def timed_over_pool(fn):
        for _ in range(3):
            for l in pool:
                fn(l)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            for l in pool:
                fn(l)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (10 * n_pool)

    xq32 = torch.randint(-127, 128, (32, Kd), dtype=torch.int8, device=dev)
    sx32 = torch.rand(32, device=dev)
    Y32 = torch.empty((32, Nd), dtype=torch.bfloat16, device=dev)
    us32 = timed_over_pool(lambda l: w2.matmul_a8(l["gate_up"], Kd, Nd, G, xq32, sx32, out=Y32))
    X16 = torch.randn(1, Kd, device=dev).to(torch.bfloat16)
    Y16 = torch.empty((1, Nd), dtype=torch.bfloat16, device=dev)
    us16g = timed_over_pool(lambda l: w2.matmul_a16(l["gate_up"], Kd, Nd, G, X16, out=Y16))
    out["other_paths"] = {"note": "eager launches (host launch cost included), gate+up 4096x28672 over the pool",
                          "w2a8_M32_us": round(us32, 2),
                          "w2a8_M32_GBps": round(algorithmic_bytes(32, Kd, Nd) / us32 / 1e3, 1),
                          "w2a16_M1_us": round(us16g, 2),
                          "w2a16_M1_GBps": round((Kd * Nd // 4 + (Kd // G) * Nd * 2 + 2 * Kd + 2 * Nd) / us16g / 1e3, 1)}

    # ---- the CPU oracle, timed as it stands on the host cores, on the same layer
    if not args.no_cpu_baseline:
        import oracle
        best = None
        for _ in range(10):
            t = time.perf_counter()
            for name in shapes:
                codes, scales, X = host[name]
                oq, osx, _ = oracle.quantize_rows(X, G, want_gsum=False)
                oracle.matmul_a8(codes, scales, G, 0, oq, osx)
            dt = time.perf_counter() - t
            best = dt if best is None else min(best, dt)
        out["cpu_baseline"] = {"value": round(step_bytes / best / 1e9, 3), "unit": "GB/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "the full step (all four projections of the layer, M=1), "
                                         "best of 10 runs; %.3f s per step" % best}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
