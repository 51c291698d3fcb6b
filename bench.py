#!/usr/bin/env python3
"""Benchmark of the operator hot path on one MI355X.

One "step" is one pass over the six operator calls of the workload (GMM 512^3, C2D,
ConvLayer, TBG, DEP, stride-2 C2D; shapes and seeds in paper_2006_06762_amd/inputs.py),
all inputs resident in HBM.  Prints ONE JSON line:

  value      whole-step fp32 throughput in TFLOP/s (sum of the operators' algorithmic
             FLOPs / step time), buffers rotated between steps so that a step does not
             find its inputs in the 256 MB Infinity Cache of the previous one; the K timed
             steps are replayed from a HIP graph of up to 48 steps (--eager: issued from Python);
             defaults K = 1000, W = 50 (a fifth of a second of GPU time);
  per_op     every operator's own launch time (HIP events on the launch stream around a
             replayed HIP graph of 48 launches), warm (same buffers) and cold (24 rotating
             buffer sets), TFLOP/s against the 157.3 TFLOP/s fp32 MFMA peak and GB/s
             against 8 TB/s; us_cold_eager is the same launch issued from Python;
  overlapped the same step with its independent operators on three streams of one HIP graph
             (forked and joined every step): ms_per_step and TFLOP/s beside `value`, which
             stays the one-stream figure; --no-overlap skips it;
  roofline   the dominant kernel (the implicit-GEMM convolution on its largest launch);
  cpu_baseline  the fp64 CPU oracle timed on the host cores on a bounded sample.

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--eager] [--no-overlap]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_F32_TFLOPS = 157.3      # 256 CU x 2.4 GHz x 256 flop/clk/CU
PEAK_HBM_GBS = 8000.0
METRIC = "achieved TFLOP/s and % of fp32 MFMA peak per operator; DEP HBM GB/s"
# the paper's own headline figures, printed beside the throughput as context (other hardware,
# other baselines: not a target and not comparable with `value`)
PAPER_CONTEXT = {
    "source": "arXiv 2006.06762, abstract and Sec. 7.3",
    "claim": "speed-up of the generated programs over the prior state of the art, up to",
    "intel_cpu": 3.8, "arm_cpu": 2.6, "nvidia_gpu": 1.7, "unit": "x",
}
MIN_TIMED_MS = 50.0               # the timed region lasts at least this long, whatever --steps is


def conv_flops(s):
    return 2.0 * s.N * s.K * s.OH * s.OW * s.C * s.R * s.S


def conv_bytes(s):
    return 4.0 * (s.N * s.C * s.H * s.W + s.K * s.C * s.R * s.S + s.N * s.K * s.OH * s.OW)


def workload_table(I):
    """Algorithmic FLOPs and compulsory bytes (each tensor once) per operator call."""
    g, t, d = I.GMM, I.TBG, I.DEP
    return {
        "GMM": (2.0 * g.M * g.N * g.K, 4.0 * (g.M * g.K + g.K * g.N + g.M * g.N), "mfma"),
        "C2D": (conv_flops(I.C2D), conv_bytes(I.C2D), "mfma"),
        "ConvLayer": (conv_flops(I.CONVLAYER), conv_bytes(I.CONVLAYER) + 4.0 * 4 * I.CONVLAYER.K, "mfma"),
        "TBG": (2.0 * t.B * t.H * t.S * t.S * t.D, 4.0 * (2 * t.B * t.S * t.H * t.D + t.B * t.H * t.S * t.S),
                "mfma"),
        "DEP": (2.0 * d.N * d.C * d.OH * d.OW * 9, 4.0 * (2 * d.N * d.C * d.H * d.W + d.C * 9), "hbm"),
        "C2D_S2": (conv_flops(I.C2D_S2), conv_bytes(I.C2D_S2), "mfma"),
        # TBS = TBG with the row softmax fused in: the matmul's flops (the softmax's ~5 S^2 per
        # head are not counted), the same compulsory bytes
        "TBS": (2.0 * t.B * t.H * t.S * t.S * t.D, 4.0 * (2 * t.B * t.S * t.H * t.D + t.B * t.H * t.S * t.S),
                "mfma"),
        "C2D_packed": (conv_flops(I.C2D), conv_bytes(I.C2D), "mfma"),
        "ConvLayer_packed": (conv_flops(I.CONVLAYER), conv_bytes(I.CONVLAYER) + 4.0 * 4 * I.CONVLAYER.K, "mfma"),
        "C2D_S2_packed": (conv_flops(I.C2D_S2), conv_bytes(I.C2D_S2), "mfma"),
    }


# measured on their own, not part of the step: the full TBS, and the three convolution launches
# with pre-packed weights (anr_conv2d_pack_weights; the packing itself is done once, untimed)
EXTRA_OPS = ("TBS", "C2D_packed", "ConvLayer_packed", "C2D_S2_packed")
PACKED_OF = {"C2D_packed": "C2D", "ConvLayer_packed": "ConvLayer", "C2D_S2_packed": "C2D_S2"}


class OpSet:
    """Device tensors of one buffer set and the six launches over them."""

    def __init__(self, anr, I, torch, host):
        self.anr = anr
        dev = lambda a: torch.from_numpy(a).cuda()
        self.t = {}
        for name in I.CONFIG_NAMES:
            cfg = host[name]
            self.t[name] = {k: dev(v) for k, v in cfg.items() if isinstance(v, np.ndarray)}
        e = lambda *shape: torch.empty(shape, dtype=torch.float32, device="cuda")
        s = I.C2D
        self.t["GMM"]["C"] = e(I.GMM.M, I.GMM.N)
        self.t["C2D"]["y"] = e(s.N, s.K, s.OH, s.OW)
        s = I.CONVLAYER
        self.t["ConvLayer"]["y"] = e(s.N, s.K, s.OH, s.OW)
        self.t["TBG"]["out"] = e(I.TBG.B, I.TBG.H, I.TBG.S, I.TBG.S)
        s = I.DEP
        self.t["DEP"]["y"] = e(s.N, s.C, s.OH, s.OW)
        s = I.C2D_S2
        self.t["C2D_S2"]["y"] = e(s.N, s.K, s.OH, s.OW)
        self.I = I
        self.packs = {}

    def pack(self, name):
        """Descriptor and pack of a convolution's constants, made on first use."""
        if name not in self.packs:
            t, s = self.t[name], {"C2D": self.I.C2D, "ConvLayer": self.I.CONVLAYER, "C2D_S2": self.I.C2D_S2}[name]
            bn = [t[k] for k in ("gamma", "beta", "mean", "var")] if name == "ConvLayer" else None
            self.packs[name] = self.anr.conv2d_pack_weights((s.N, s.C, s.H, s.W), t["w"], s.stride, s.pad, bn=bn,
                                                            eps=self.I.BN_EPS)
        return self.packs[name]

    def run(self, name):
        if name in PACKED_OF:
            base = PACKED_OF[name]
            d, pack = self.pack(base)
            t = self.t[base]
            fn = self.anr.conv_bn_relu_packed if base == "ConvLayer" else self.anr.conv2d_packed
            fn(d, t["x"], pack, t["y"])
            return
        a, t, I = self.anr, self.t["TBG" if name == "TBS" else name], self.I
        if name == "GMM":
            a.gemm(t["A"], t["B"], t["C"])
        elif name == "C2D":
            a.conv2d(t["x"], t["w"], t["y"], I.C2D.stride, I.C2D.pad)
        elif name == "ConvLayer":
            a.conv_bn_relu(t["x"], t["w"], t["gamma"], t["beta"], t["mean"], t["var"], I.BN_EPS, t["y"],
                           I.CONVLAYER.stride, I.CONVLAYER.pad)
        elif name == "TBG":
            a.tbg(t["q"], t["k"], t["out"])
        elif name == "TBS":
            a.tbs(t["q"], t["k"], t["out"])
        elif name == "DEP":
            a.dwconv(t["x"], t["w"], t["y"], I.DEP.stride, I.DEP.pad)
        elif name == "C2D_S2":
            a.conv2d(t["x"], t["w"], t["y"], I.C2D_S2.stride, I.C2D_S2.pad)
        else:
            raise KeyError(name)

    def output(self, name):
        t = self.t["TBG" if name == "TBS" else PACKED_OF.get(name, name)]
        return t.get("y", t.get("C", t.get("out")))

    def step(self):
        for name in self.I.CONFIG_NAMES:
            self.run(name)


def time_launches(torch, fn, reps):
    """Average time of one call of fn in microseconds, by HIP events on the launch stream."""
    start = torch.cuda.Event(enable_timing=True)
    end = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for i in range(reps):
        fn(i)
    end.record()
    torch.cuda.synchronize()
    return start.elapsed_time(end) * 1000.0 / reps


def time_graph(torch, fn, launches, replays=10):
    """Average time of one call of fn in microseconds when `launches` calls are captured in one
    HIP graph (no host launch overhead between kernels) and the graph is replayed."""
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        for i in range(launches):       # warm-up on the capture stream, outside the capture
            fn(i)
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(launches):
                fn(i)
        graph.replay()
        stream.synchronize()
        start = torch.cuda.Event(enable_timing=True)
        end = torch.cuda.Event(enable_timing=True)
        start.record(stream)
        for _ in range(replays):
            graph.replay()
        end.record(stream)
        stream.synchronize()
    torch.cuda.current_stream().wait_stream(stream)
    return start.elapsed_time(end) * 1000.0 / (launches * replays)


# Independent operators of a step on separate streams: the stride-2 convolution alone, the two
# stride-1 convolutions one after the other, the three short kernels one after the other.  The
# convolution kernels hold one work-group per CU on 224 of the 256 CUs and leave a SIMD idle at
# every barrier; kernels of other streams run in those gaps.
OVERLAP_PLAN = (("C2D_S2",), ("C2D", "ConvLayer"), ("GMM", "TBG", "DEP"))


def overlapped_steps(torch, sets, group, steps):
    """Milliseconds per step when the step's six launches are issued on three streams (forked from
    and joined to the main stream in every step) inside one HIP graph of `group` steps."""
    main = torch.cuda.Stream()
    side = [torch.cuda.Stream() for _ in OVERLAP_PLAN[1:]]     # default priority, like every stream here
    main.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(main):
        with torch.cuda.graph(graph, stream=main):
            for i in range(group):
                s = sets[i % 4]
                for st in side:
                    st.wait_stream(main)
                for ops, st in zip(OVERLAP_PLAN[1:], side):
                    with torch.cuda.stream(st):
                        for n in ops:
                            s.run(n)
                for n in OVERLAP_PLAN[0]:
                    s.run(n)
                for st in side:
                    main.wait_stream(st)
        graph.replay()                           # untimed: uploads the graph
        main.synchronize()
        torch.cuda.synchronize()
        replays = max(1, steps // group)
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        main.synchronize()
        wall = time.perf_counter() - t0
    torch.cuda.current_stream().wait_stream(main)
    return wall * 1000.0 / (replays * group)


def shape_list(anr, I, torch):
    """Launch times of every Appendix C shape at batch 1 and 16 (operator and subgraph benchmarks,
    Sec. 7.1 and 7.2).  Timing only: values are uniform random numbers drawn on the device."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(I.SEED_BASE)
    rnd = lambda *shape: torch.rand(shape, generator=gen, device="cuda", dtype=torch.float32) * 2 - 1
    emp = lambda *shape: torch.empty(shape, device="cuda", dtype=torch.float32)
    rows = []
    for op in ("GMM", "C2D", "DEP", "ConvLayer", "TBS", "GRP", "DIL", "NRM"):
        for fields in I.APPENDIX_C[op]:
            for batch in I.BATCHES:
                s = I.appendix_shape(op, fields, batch) if op != "NRM" else fields
                if s is None:          # a record that cannot be built (3 channels in 4 groups)
                    continue
                if op == "NRM":
                    n_, m_ = fields
                    flops = 2.0 * batch * n_ * m_
                    nbytes = 4.0 * batch * n_ * m_
                    mk = lambda: (rnd(batch, n_, m_), emp(batch))
                    run = lambda t: anr.nrm(t[0], t[1])
                elif op == "GMM":
                    flops = 2.0 * s.batch * s.M * s.N * s.K
                    nbytes = 4.0 * s.batch * (s.M * s.K + s.K * s.N + s.M * s.N)
                    mk = lambda: (rnd(s.batch, s.M, s.K), rnd(s.batch, s.K, s.N), emp(s.batch, s.M, s.N))
                    run = lambda t: anr.gemm(t[0], t[1], t[2])
                elif op == "TBS":
                    flops = 2.0 * s.B * s.H * s.S * s.S * s.D
                    nbytes = 4.0 * (2 * s.B * s.S * s.H * s.D + s.B * s.H * s.S * s.S)
                    mk = lambda: (rnd(s.B, s.S, s.H, s.D), rnd(s.B, s.S, s.H, s.D), emp(s.B, s.H, s.S, s.S))
                    run = lambda t: anr.tbs(t[0], t[1], t[2])
                else:
                    dw = op == "DEP"
                    cin = 1 if dw else s.C // s.groups
                    flops = 2.0 * s.N * s.K * s.OH * s.OW * cin * s.R * s.S
                    nbytes = 4.0 * (s.N * s.C * s.H * s.W + s.K * cin * s.R * s.S + s.N * s.K * s.OH * s.OW)
                    if op == "ConvLayer":
                        mk = lambda: (rnd(s.N, s.C, s.H, s.W), rnd(s.K, s.C, s.R, s.S) * 0.05, emp(s.N, s.K, s.OH, s.OW),
                                      rnd(s.K) * 0.5 + 1, rnd(s.K) * 0.1, rnd(s.K) * 0.1, rnd(s.K) * 0.75 + 1.25)
                        run = lambda t: anr.conv_bn_relu(t[0], t[1], t[3], t[4], t[5], t[6], I.BN_EPS, t[2],
                                                         s.stride, s.pad)
                    elif dw:
                        mk = lambda: (rnd(s.N, s.C, s.H, s.W), rnd(s.C, 1, s.R, s.S) * 0.05, emp(s.N, s.K, s.OH, s.OW))
                        run = lambda t: anr.dwconv(t[0], t[1], t[2], s.stride, s.pad)
                    else:
                        mk = lambda: (rnd(s.N, s.C, s.H, s.W), rnd(s.K, cin, s.R, s.S) * 0.05, emp(s.N, s.K, s.OH, s.OW))
                        run = lambda t: anr.conv2d(t[0], t[1], t[2], s.stride, s.pad, dil=s.dil, groups=s.groups)
                # enough buffer sets that a launch does not find its data in the 256 MB Infinity Cache:
                # 600 MB in rotation where 24 sets reach that (at 300 MB the cache still served part of
                # a 25 MB operator); the small shapes stay cache-resident whatever the count
                nsets = int(min(24, max(2, -(-600e6 // nbytes))))
                sets = [mk() for _ in range(nsets)]
                for t in sets:
                    run(t)
                torch.cuda.synchronize()
                warm = time_graph(torch, lambda i: run(sets[0]), 2 * nsets)
                cold = time_graph(torch, lambda i: run(sets[i % nsets]), 2 * nsets)
                # the shape's own roofline: the larger of its matrix time and its traffic time
                t_mfma, t_hbm = flops / PEAK_MFMA_F32_TFLOPS / 1e6, nbytes / PEAK_HBM_GBS / 1e3     # microseconds
                rows.append({"op": op, "shape": list(fields), "batch": batch, "us_warm": warm, "us_cold": cold,
                             "tflops_cold": flops / cold / 1e6, "gbs_cold": nbytes / cold / 1e3,
                             "frac_mfma_peak_cold": flops / cold / 1e6 / PEAK_MFMA_F32_TFLOPS,
                             "frac_hbm_peak_cold": nbytes / cold / 1e3 / PEAK_HBM_GBS, "buffer_sets": nsets,
                             "bound": "mfma" if t_mfma >= t_hbm else "hbm",
                             "roofline_us": max(t_mfma, t_hbm), "frac_own_roofline_cold": max(t_mfma, t_hbm) / cold})
                del sets
    return rows


def trace_summary(db_path):
    """Per-kernel launch statistics from the rocpd database that `rocprofv3 --kernel-trace`
    writes: calls, average / minimum / median duration in microseconds."""
    import collections
    import re
    import sqlite3
    import statistics
    con = sqlite3.connect(db_path)
    per = collections.defaultdict(list)
    for name, start, end in con.execute("select name, start, end from kernels"):
        per[name].append(end - start)
    lines = ["%-90s %6s %10s %10s %10s" % ("kernel", "calls", "avg_us", "min_us", "med_us")]
    for name, v in sorted(per.items(), key=lambda kv: -sum(kv[1])):
        short = re.sub(r"\(anonymous namespace\)::", "", name)[:90]
        lines.append("%-90s %6d %10.2f %10.2f %10.2f" % (short, len(v), sum(v) / len(v) / 1e3, min(v) / 1e3,
                                                         statistics.median(v) / 1e3))
    return "\n".join(lines)


def oracle_reference(I, host, name):
    import oracle
    name = PACKED_OF.get(name, name)
    c = host["TBG" if name == "TBS" else name]
    s = c["shape"]
    if name == "GMM":
        return oracle.gemm(c["A"], c["B"])
    if name in ("C2D", "C2D_S2"):
        return oracle.conv2d(c["x"], c["w"], s.stride, s.pad)
    if name == "ConvLayer":
        return oracle.conv_bn_relu(c["x"], c["w"], c["gamma"], c["beta"], c["mean"], c["var"], c["eps"],
                                   s.stride, s.pad)
    if name == "TBG":
        return oracle.tbg(c["q"], c["k"])
    if name == "TBS":
        return oracle.tbs(c["q"], c["k"])
    if name == "DEP":
        return oracle.dwconv(c["x"], c["w"], s.stride, s.pad)
    raise KeyError(name)


def cpu_baseline(I, host, table):
    """Time the fp64 oracle, as it stands, on the host cores: whole passes over the step (all six
    operators at full size), repeated until two seconds of wall time (some 30 core-seconds) have
    gone by.  Also returns the references for the parity check."""
    import oracle
    cores = oracle.max_threads()
    refs = {}
    passes, dt = 0, 0.0
    while passes == 0 or dt < 2.0:
        t0 = time.perf_counter()
        for name in I.CONFIG_NAMES:
            refs[name] = oracle_reference(I, host, name)
        dt += time.perf_counter() - t0
        passes += 1
    flops = sum(table[n][0] for n in I.CONFIG_NAMES)
    return refs, {
        "value": flops * passes / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
        "seconds": dt, "passes": passes,
        "sample": "%d full steps (all six operator calls at full size, %.2f GFLOP each), OpenMP over the "
                  "outer loop on %d threads" % (passes, flops / 1e9, cores),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle timing and parity check (profiling runs)")
    ap.add_argument("--eager", action="store_true",
                    help="issue every timed step from Python instead of replaying a HIP graph of steps")
    ap.add_argument("--no-overlap", action="store_true",
                    help="skip the extra timing of the step with its operators on three streams (profiling runs: "
                         "keeps every kernel's launches free of other kernels)")
    ap.add_argument("--only", default=None, help="profiling aid: launch only this operator in the step")
    ap.add_argument("--cold-only", action="store_true",
                    help="profiling aid: every launch of the run reads buffers that are not in the caches (24 sets in "
                         "rotation everywhere, no warm or eager per-operator timing), so that a kernel trace of the "
                         "run holds cold launches only")
    ap.add_argument("--no-per-op", action="store_true",
                    help="profiling aid: time the step only (no per-operator timing loops, no roofline): with --only, "
                         "--cold-only and --eager every launch of the run is one cold launch of that operator's kernel, "
                         "issued on its own")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="profiling aid: run 10 plain device copies of 256 MiB (known HBM traffic for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--shape-list", action="store_true",
                    help="instead of the step, time every Appendix C shape at batch 1 and 16 and print one JSON line")
    ap.add_argument("--trace-summary", default=None, metavar="DB",
                    help="print per-kernel statistics of a rocprofv3 --kernel-trace database (no GPU needed) and exit")
    args = ap.parse_args()
    if args.trace_summary:
        print(trace_summary(args.trace_summary))
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); multi-GPU figures are not produced",
              file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    from paper_2006_06762_amd import build as hip_build
    hip_build.ensure_built()
    from paper_2006_06762_amd import binding as anr
    from paper_2006_06762_amd import inputs as I

    if args.copy_calibration:
        n = 256 << 20
        src = torch.ones(n // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_each_way": n, "copies": 10}))
        return

    if args.shape_list:
        print(json.dumps({"metric": "launch time per Appendix C shape (HIP-graph timed, warm and cold buffers)",
                          "unit": "us", "dtype": "f32", "data": "synthetic", "n_gpus": 1,
                          "peaks": {"mfma_f32_tflops": PEAK_MFMA_F32_TFLOPS, "hbm_gbs": PEAK_HBM_GBS},
                          "shapes": shape_list(anr, I, torch)}))
        return

    table = workload_table(I)
    host = {name: I.config_inputs(name) for name in I.CONFIG_NAMES}
    names = I.CONFIG_NAMES if args.only is None else (args.only,)

    # one step touches ~135 MB; 4 rotating sets keep a step from finding its data in the
    # 256 MB Infinity Cache.  A single operator's tensors are ~25 MB: with 12 sets (300 MB) the
    # cache still served part of them (TBG 8.5 us against 9.1 us with 24 or 48 sets), so 24
    NSETS = 24
    sets = [OpSet(anr, I, torch, host) for _ in range(NSETS)]

    # a whole step moves ~135 MB, so four sets in rotation keep it out of the caches; one operator
    # alone (--only) moves ~25 MB and rotates all 24
    rot = 4 if args.only is None else NSETS

    def step(i):
        s = sets[i % rot]
        for n in names:
            s.run(n)

    t0 = time.perf_counter()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    est_ms = (time.perf_counter() - t0) * 1000.0 / max(1, args.warmup)
    # K steps make one round; short runs time several rounds so that the timed region is not a
    # single graph replay of a few milliseconds
    rounds = 1 if args.warmup == 0 else max(1, int(np.ceil(MIN_TIMED_MS / max(1e-3, est_ms * args.steps))))
    # The timed K steps.  Several kernels of a step run 6-9 us, less than it takes Python to issue
    # a launch, so the GPU waits for the host now and then (about 2.5 % of a step).  By default
    # the steps are therefore captured in a HIP graph of up to 48 steps (a multiple of the 4
    # rotating buffer sets) that is replayed K // G times, the remaining K % G steps issued one by
    # one on the same stream; --eager issues all K steps from Python.
    if args.eager:
        group = 0
    elif rot == 4:
        group = (min(args.steps, 48) // 4) * 4
    else:
        group = (min(args.steps, 2 * rot) // rot) * rot
    if group and rot == 4:
        # prefer a graph length that divides K, so that no step is left over for the eager tail
        for cand in range(group, 19, -4):
            if args.steps % cand == 0:
                group = cand
                break
    if group:
        stream = torch.cuda.Stream()
        stream.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(stream):
            with torch.cuda.graph(graph, stream=stream):
                for i in range(group):
                    step(i)
            graph.replay()                       # untimed: uploads the graph
            stream.synchronize()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(rounds):
                for _ in range(args.steps // group):
                    graph.replay()
                for i in range(args.steps % group):
                    step(i)
            stream.synchronize()
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
        torch.cuda.current_stream().wait_stream(stream)
    else:
        t0 = time.perf_counter()
        for _ in range(rounds):
            for i in range(args.steps):
                step(i)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms_per_step = wall * 1000.0 / (args.steps * rounds)
    step_flops = sum(table[n][0] for n in names)
    value = step_flops / (ms_per_step * 1e-3) / 1e12

    # per-operator launch times
    per_op = []
    measured = tuple(names) + (EXTRA_OPS if args.only is None else ())
    if args.no_per_op:
        measured = ()
    for n in measured:
        flops, nbytes, bound = table[n]
        reps = 200
        for i in range(10):
            sets[i % NSETS if args.cold_only else 0].run(n)
        # launches captured in a HIP graph: kernel time plus the GPU's own kernel-to-kernel gap
        cold = time_graph(torch, lambda i: sets[i % NSETS].run(n), 2 * NSETS)
        if args.cold_only:
            warm = eager = float("nan")
        else:
            warm = time_graph(torch, lambda i: sets[0].run(n), 2 * NSETS)
            # the same launches issued one by one from Python (adds host launch overhead)
            eager = time_launches(torch, lambda i: sets[i % NSETS].run(n), reps)
        rec = {"op": n, "bound": bound, "flops": flops, "bytes": nbytes,
               "us_warm": warm, "us_cold": cold, "us_cold_eager": eager,
               "tflops_warm": flops / warm / 1e6, "tflops_cold": flops / cold / 1e6,
               "gbs_warm": nbytes / warm / 1e3, "gbs_cold": nbytes / cold / 1e3}
        rec["frac_mfma_peak_warm"] = rec["tflops_warm"] / PEAK_MFMA_F32_TFLOPS
        rec["frac_mfma_peak_cold"] = rec["tflops_cold"] / PEAK_MFMA_F32_TFLOPS
        rec["frac_hbm_peak_cold"] = rec["gbs_cold"] / PEAK_HBM_GBS
        rec["in_step"] = n in names
        per_op.append(rec)

    if not per_op:
        print(json.dumps({"metric": METRIC, "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
                          "warmup": args.warmup, "ms_per_step": ms_per_step, "dtype": "f32", "data": "synthetic",
                          "config": {"workload": "only " + str(args.only), "buffer_sets_rotated": rot,
                                     "timed_steps": args.steps * rounds}}))
        return
    by = {r["op"]: r for r in per_op}
    dom = by.get("C2D_S2") or per_op[0]
    # HBM traffic per launch is a stored figure (two rocprofv3 --pmc runs, kept under profiles/),
    # not something this run measures
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(dom["op"])
        except Exception:
            traffic = None
    traffic_source = "stored: profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE)" if traffic else None
    # the kernel behind each operator's benchmark launch (with --only, the roofline is that operator's)
    kernels = {"GMM": "gemm_tile32_ksplit_kernel", "C2D": "conv_igemm_kernel", "ConvLayer": "conv_igemm_kernel",
               "C2D_S2": "conv_igemm_kernel", "TBG": "tbg_tile64_kernel", "TBS": "tbs_rows32_kernel",
               "DEP": "dwconv3x3_stream_kernel"}
    if dom["bound"] == "hbm":
        roofline = {
            "kernel": "%s (%s launch)" % (kernels.get(dom["op"], "?"), dom["op"]), "bound": "hbm",
            "achieved": dom["gbs_cold"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": dom["gbs_cold"] / PEAK_HBM_GBS, "traffic": traffic, "traffic_source": traffic_source,
            "launch_us": dom["us_cold"],
        }
    else:
        roofline = {
            "kernel": "%s (%s launch)" % (kernels.get(dom["op"], "?"), dom["op"]), "bound": "mfma",
            "achieved": dom["tflops_cold"], "peak": PEAK_MFMA_F32_TFLOPS, "unit": "TFLOP/s",
            "frac": dom["tflops_cold"] / PEAK_MFMA_F32_TFLOPS, "traffic": traffic,
            "traffic_source": traffic_source, "launch_us": dom["us_cold"],
        }

    out = {
        "metric": METRIC, "value": value, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "one step = GMM 512^3 + C2D N16 64->64 56^2 3x3 + ConvLayer N16 128->128 28^2 "
                               "3x3+BN+ReLU + TBG B16 S128 H12 D64 + DEP N16 C256 28^2 3x3 + C2D N16 256->512 "
                               "28^2 3x3 s2 (all BASELINE configs, fp32)" if args.only is None
                   else "only " + args.only,
                   "step_gflop": step_flops / 1e9, "buffer_sets_rotated": rot,
                   "steps_per_graph_replay": group, "timed_rounds_of_k_steps": rounds,
                   "timed_steps": args.steps * rounds},
        "paper_context": PAPER_CONTEXT,
        "roofline": roofline,
        "peaks": {"mfma_f32_tflops": PEAK_MFMA_F32_TFLOPS, "hbm_gbs": PEAK_HBM_GBS},
        "per_op": per_op,
    }

    if group and args.only is None and not args.no_overlap:
        # the same step with independent operators overlapped; outputs must be bit-identical to the
        # one-stream step's (same kernels on the same inputs)
        seq = {}
        sets[0].step()
        torch.cuda.synchronize()
        for n in names:
            seq[n] = sets[0].output(n).clone()
            sets[0].output(n).zero_()
        ms_overlap = overlapped_steps(torch, sets, group, args.steps)
        torch.cuda.synchronize()
        out["overlapped"] = {
            "ms_per_step": ms_overlap, "value": step_flops / (ms_overlap * 1e-3) / 1e12, "unit": "TFLOP/s",
            "streams": [list(ops) for ops in OVERLAP_PLAN], "steps_per_graph_replay": group,
            "outputs_identical": all(bool(torch.equal(seq[n], sets[0].output(n))) for n in names),
            "note": "same six launches per step, independent operators on three streams of one HIP graph, "
                    "joined every step; `value` above is the one-stream step",
        }

    if not args.no_cpu_baseline and args.only is None:
        refs, base = cpu_baseline(I, host, table)
        out["cpu_baseline"] = base
        errs = {}
        for n in EXTRA_OPS:
            refs[n] = oracle_reference(I, host, n)      # outside the timed oracle pass
        for n in measured:
            sets[0].run(n)
            got = sets[0].output(n).cpu().numpy().astype(np.float64)
            errs[n] = float(np.max(np.abs(got - refs[n]) / np.maximum(1.0, np.abs(refs[n]))))
        out["max_rel_err_vs_oracle"] = errs
        out["parity_ok"] = all(e <= 1e-4 for e in errs.values())
    print(json.dumps(out))
    if out.get("parity_ok") is False:
        print("bench.py: parity against the oracle FAILED: %s" % out["max_rel_err_vs_oracle"], file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
