#!/usr/bin/env python3
"""Headline benchmark: the discount task (paper Fig. 1 / Query 1) at M = N = K = 8192, fp32,
on one MI355X, through the library's C ABI.

A step is one amulet_mmlike_f32 call (the whole hot path: operand staging, per-product g,
k-reduction, R += write-back) on synthetic retail-style inputs already resident in HBM.
Prints one JSON line: effective GFLOP/s = 2MNK/t (the paper's SPR times two), the kernel's
share of the fp32 vector peak ("roofline"), and the CPU oracle timed on a bounded sample of
the same workload ("cpu_baseline", a reported baseline only).  The default run then adds a
`configs` array to the same line: every other named workload (cfg0-cfg4, Query 3, the fp64
variants) as a short leg of its own after the headline's timed region, with its kernel time,
roofline fraction, sampled parity against the oracle and, for the identity task, the library
SGEMM on the same buffers.  The exit status is 3 when any sampled parity check fails.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peak used as the roofline denominator: fp32 vector 157.3 TFLOP/s
# = 256 CU x 2.4 GHz x 128 lanes/clk/CU x 2 flop (one FMA per lane-operation).
FP32_VECTOR_PEAK_TFLOPS = 157.3
# The same units counted in lane-operations: a predicate task spends several VALU
# lane-operations per product (discount: multiply, compare, select, FMA), so its ceiling
# in the metric's 2-flop-per-product convention is 2 x 78.6e12 / ops.
VALU_LANE_OPS_PER_S = 256 * 128 * 2.4e9
# (count_gt: multiply, subtract, shift, and one three-input add per two products of an accumulator)
VALU_OPS_PER_PRODUCT = {"discount": 4, "boost": 4, "count_gt": 3.5, "identity": 1}


class ShaderClock:
    """Samples the GPU's current shader clock (the starred line of the driver's pp_dpm_sclk file)
    from a thread while a timed region runs.  The published peaks are at 2.4 GHz; under a full
    vector-ALU load the chip holds less (power), and the sample says how much.  Context only:
    `frac` stays against the published peak.  Reports None where the file cannot be read."""

    def __init__(self, period_s=0.02):
        import glob
        self.paths = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.period_s = period_s
        self.samples = []
        self._stop = None
        self._thread = None

    def _read(self):
        for path in self.paths:
            try:
                with open(path) as f:
                    for line in f:
                        if "*" in line:
                            digits = "".join(c for c in line.split(":", 1)[-1] if c.isdigit())
                            if digits:
                                return int(digits)
            except OSError:
                continue
        return None

    def __enter__(self):
        import threading
        self._stop = threading.Event()

        def loop():
            while not self._stop.is_set():
                mhz = self._read()
                if mhz:
                    self.samples.append(mhz)
                self._stop.wait(self.period_s)

        if self.paths:
            self._thread = threading.Thread(target=loop, daemon=True)
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        if self._thread is not None:
            self._thread.join()
        return False

    def median_mhz(self):
        # (the first samples may predate the first launch: idle clock; the median of a region of
        # tens of milliseconds or more is the loaded clock)
        if len(self.samples) < 5:    # a region of less than about 100 ms: too few samples to say
            return None
        return sorted(self.samples)[len(self.samples) // 2]


INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense int8 matrix peak, 5.0 POP/s
FP64_VECTOR_PEAK_TFLOPS = 78.6  # MI355X fp64 vector peak


def bench_count_i8(args, am, torch, np, spec, A, B) -> dict:
    """Secondary line: the int8 join count (R += A.B, exact) on the matrix cores."""
    M, N, K = spec["M"], spec["N"], spec["K"]
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dR = torch.zeros(M, N, dtype=torch.int32, device="cuda")
    T = am.AMULET_TASK_COUNT_I8
    # (--i8-assign: the launches that are timed, traced or counted are of the R = form)
    count = (lambda a, b, r: am.amulet_count_i8_assign(a, b, r)) if args.i8_assign else am.amulet_count_i8
    if args.traffic_probe:
        # for rocprofv3 --pmc runs: one plain 256 MiB device copy (known HBM bytes: the counter
        # calibration), then --steps launches of the kernel
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        if not args.no_tune:
            am.amulet_tune(T, M, N, K)
        for _ in range(args.steps):
            count(dA, dB, dR)
        torch.cuda.synchronize()
        print("traffic probe done: 1 copy of %d bytes, %d launches of %s" %
              (src.numel() * 4, args.steps, am.amulet_shape_name(T, am.amulet_selected_shape(T, M, N, K))))
        return {}
    t0 = time.perf_counter()
    shape = am.amulet_selected_shape(T, M, N, K) if args.no_tune else am.amulet_tune(T, M, N, K)
    tune_s = time.perf_counter() - t0
    for _ in range(args.warmup):
        count(dA, dB, dR)
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    with ShaderClock() as sclk:
        w0 = time.perf_counter()
        for i in range(args.steps):
            starts[i].record()
            count(dA, dB, dR)
            stops[i].record()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - w0) * 1e3 / args.steps
    sclk_mhz = sclk.median_mhz()
    kern_ms = [s.elapsed_time(e) for s, e in zip(starts, stops)]
    kernel_ms_avg = sum(kern_ms) / args.steps
    kernel_ms_median = sorted(kern_ms)[len(kern_ms) // 2]
    ops = 2.0 * M * N * K
    achieved = ops / (kernel_ms_avg * 1e-3) / 1e12
    # The same join written instead of accumulated (R = A.B, amulet_count_i8_assign: the workload's
    # own definition; the write-back does not read R).  Reported beside the += form, which stays
    # the leg's figure; R starts full of another value and is checked against the same sample.
    Ra = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    for _ in range(args.warmup):
        am.amulet_count_i8_assign(dA, dB, Ra)
    torch.cuda.synchronize()
    for i in range(args.steps):
        starts[i].record()
        am.amulet_count_i8_assign(dA, dB, Ra)
        stops[i].record()
    torch.cuda.synchronize()
    assign_ms = sum(s.elapsed_time(e) for s, e in zip(starts, stops)) / args.steps
    assign_tops = ops / (assign_ms * 1e-3) / 1e12
    # what the matrix cores sustain on this instruction with nothing around it (the clock
    # drops under matrix-core load, so this is below the nominal peak)
    probe_tops = 2.0 * am.amulet_probe_mfma_i8(4) / 1e12
    cpu, exact = None, None
    if args.cpu_rows > 0:
        import oracle
        rows = np.sort(np.random.Generator(np.random.PCG64(99)).choice(M, min(4 * args.cpu_rows, M), replace=False))
        Rz = torch.zeros(M, N, dtype=torch.int32, device="cuda")
        am.amulet_count_i8(dA, dB, Rz)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        R_ref, threads = oracle.count_i8(np.ascontiguousarray(A[rows]), B)
        cpu_s = time.perf_counter() - c0
        exact = bool(np.array_equal(Rz[torch.from_numpy(rows).cuda()].cpu().numpy(), R_ref)) and \
            bool(np.array_equal(Ra[torch.from_numpy(rows).cuda()].cpu().numpy(), R_ref))
        cpu = {"value": round(2.0 * len(rows) * N * K / cpu_s / 1e9, 3), "unit": "GOP/s (2MNK/t)", "cores": threads,
               "kind": "oracle", "sample": "%d whole rows of the %dx%dx%d workload, %.1f s" % (len(rows), M, N, K, cpu_s)}
    return {
        "metric": "effective GOP/s (2MNK/t), int8 join count %dx%dx%d" % (M, N, K),
        "value": round(ops / (ms_per_step * 1e-3) / 1e9, 1), "unit": "GOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": args.workload, "task": "count_i8", "M": M, "N": N, "K": K,
                   "tile_shape": am.amulet_shape_name(T, shape), "tuned": not args.no_tune,
                   "tune_seconds": round(tune_s, 3)},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": round(achieved / INT8_MFMA_PEAK_TOPS, 4), "traffic": None,
                     "kernel_ms_avg": round(kernel_ms_avg, 4), "kernel_ms_median": round(kernel_ms_median, 4),
                     "shader_clock_mhz": sclk_mhz,
                     "compulsory_bytes": M * K + K * N + 8 * M * N,
                     "mfma_probe_tops": round(probe_tops, 1),
                     "frac_of_mfma_probe": round(achieved / probe_tops, 4),
                     "assign_form": {"kernel_ms_avg": round(assign_ms, 4), "achieved": round(assign_tops, 2),
                                     "frac": round(assign_tops / INT8_MFMA_PEAK_TOPS, 4),
                                     "compulsory_bytes": M * K + K * N + 4 * M * N}},
        "cpu_baseline": cpu, "bit_exact_on_sample": exact,
        "parity_ok": None if exact is None else bool(exact)}


def bench_f64(args, am, torch, np, wl, spec, A, B, P) -> dict:
    """Secondary line: a task in the paper's own element type (fp64) on the vector ALU."""
    task, M, N, K = spec["task"], spec["M"], spec["N"], spec["K"]
    tname = wl.TASK_NAMES[task]
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    th = torch.from_numpy(P[0]).cuda() if P is not None else None
    dis = torch.from_numpy(P[1]).cuda() if (P is not None and P.shape[0] > 1) else None
    dR = torch.zeros(M, N, dtype=torch.float64, device="cuda")
    def time_library_dgemm():
        for _ in range(args.warmup):
            torch.mm(dA, dB)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            torch.mm(dA, dB)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    lib_before = time_library_dgemm() if tname == "identity" else None
    for _ in range(args.warmup):
        am.amulet_mmlike_f64(task, dA, dB, th, dis, dR)
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    with ShaderClock() as sclk:
        w0 = time.perf_counter()
        for i in range(args.steps):
            starts[i].record()
            am.amulet_mmlike_f64(task, dA, dB, th, dis, dR)
            stops[i].record()
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - w0) * 1e3 / args.steps
    sclk_mhz = sclk.median_mhz()
    kern_ms = [s.elapsed_time(e) for s, e in zip(starts, stops)]
    kernel_ms_avg = sum(kern_ms) / args.steps
    kernel_ms_median = sorted(kern_ms)[len(kern_ms) // 2]
    flops = 2.0 * M * N * K
    achieved = flops / (kernel_ms_avg * 1e-3) / 1e12
    # issue slots per product (discount: mul, compare into the execution mask, masked mul, add)
    ops = {"identity": 1, "discount": 4, "boost": 4, "count_gt": 4}[tname]
    lib_ratio = None
    if tname == "identity":   # the library DGEMM on the same buffers, timed before and after, faster run kept
        lib_ms = min(lib_before, time_library_dgemm())
        lib_ratio = {"library_dgemm_ms": round(lib_ms, 4), "ours_over_library_rate": round(lib_ms / kernel_ms_avg, 4)}
    cpu, parity = None, None
    if args.cpu_rows > 0:
        import oracle
        rows = np.sort(np.random.Generator(np.random.PCG64(99)).choice(M, min(args.cpu_rows, M), replace=False))
        Rz = torch.zeros(M, N, dtype=torch.float64, device="cuda")
        am.amulet_mmlike_f64(task, dA, dB, th, dis, Rz)
        torch.cuda.synchronize()
        R_rows = Rz[torch.from_numpy(rows).cuda()].cpu().numpy()
        c0 = time.perf_counter()
        R_ref, ab, threads = oracle.mmlike_f64_general(task, np.ascontiguousarray(A[rows]), B,
                                                       None if P is None else P[0],
                                                       None if (P is None or P.shape[0] < 2) else P[1])
        cpu_s = time.perf_counter() - c0
        cpu = {"value": round(2.0 * len(rows) * N * K / cpu_s / 1e9, 3), "unit": "GFLOP/s (2MNK/t)",
               "cores": threads, "kind": "oracle",
               "sample": "%d whole rows of the %dx%dx%d workload, %.1f s" % (len(rows), M, N, K, cpu_s)}
        parity = float(np.max(np.abs(R_rows - R_ref) / np.where(ab > 0, ab, 1.0)))
    return {
        "metric": "effective GFLOP/s (2MNK/t), %s task %dx%dx%d fp64" % (tname, M, N, K),
        "value": round(flops / (ms_per_step * 1e-3) / 1e9, 1), "unit": "GFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": args.workload, "task": tname, "M": M, "N": N, "K": K,
                   "tile_shape": ("mfma_f64_64x64_dma4" if am.amulet_selected_shape_f64(task, M, N, K) % 2 == 0
                                  else "mfma_f64_128x128_dma4") if tname == "identity" else
                   am.amulet_f64_shape_name(am.amulet_selected_shape_f64(task, M, N, K))},
        "roofline": {"bound": "mfma" if tname == "identity" else "alu", "achieved": round(achieved, 3), "peak": FP64_VECTOR_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / FP64_VECTOR_PEAK_TFLOPS, 4), "traffic": None,
                     "kernel_ms_avg": round(kernel_ms_avg, 4), "kernel_ms_median": round(kernel_ms_median, 4),
                     "shader_clock_mhz": sclk_mhz,
                     "valu_ops_per_product": ops,
                     "op_mix_ceiling_tflops": round(FP64_VECTOR_PEAK_TFLOPS / ops, 3),
                     "frac_of_op_mix_ceiling": round(achieved * ops / FP64_VECTOR_PEAK_TFLOPS, 4)},
        "cpu_baseline": cpu, "parity_worst_ratio_on_sample": parity,
        "parity_ok": None if parity is None else bool(parity <= 1e-12), "library_dgemm": lib_ratio,
        "paper_context": "AMULET Query 1 on one Xeon 6312U thread, double: SPR 7.50 = 15.0 GFLOP/s (Table 4)"}


def bench_nonsquare(args, am, torch) -> int:
    """The paper's non-square protocol (Sec. 6.4): one of M, N, K is 4096 c, another 4096 / c, the
    third 4096, c in {2, 4, 8}: 18 shapes of equal work, plus the square one.  Reports, for the
    workload's task in fp32, the rate of each shape with the operands read in place and with
    packing allowed, and mean / standard deviation / minimum over the 18.  Inputs are drawn on the
    device in the retail recipe of the headline workload (results are not checked here: parity
    of every kernel is the tests' job)."""
    import itertools
    import statistics

    task = {"discount": 1, "boost": 2, "count_gt": 3, "identity": 0}[args.nonsquare]
    gen = torch.Generator(device="cuda").manual_seed(7)

    def rate(M, N, K, packed):
        A = torch.randint(0, 10, (M, K), device="cuda", generator=gen).float()
        B = torch.rand(K, N, device="cuda", generator=gen) * 99 + 1
        th = torch.rand(N, device="cuda", generator=gen) * 400 + 100
        dis = torch.rand(N, device="cuda", generator=gen) * 0.25 + 0.05
        R = torch.zeros(M, N, device="cuda")
        ws = torch.empty(am.amulet_autopack_workspace_bytes(4, M, K), dtype=torch.uint8, device="cuda") \
            if packed else None

        def call():
            am.amulet_mmlike_f32_autopack(task, A, B, th if task else None, dis if task == 1 else None, R, ws)
        for _ in range(args.warmup):
            call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            call()
        e1.record()
        torch.cuda.synchronize()
        return 2.0 * M * N * K / (e0.elapsed_time(e1) / args.steps * 1e-3) / 1e12

    out = {"metric": "effective TFLOP/s (2MNK/t), %s task, non-square protocol, fp32" % args.nonsquare,
           "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "dtype": "f32",
           "data": "synthetic", "config": {"workload": "nonsquare_%s_4096" % args.nonsquare}}
    for packed in (False, True):
        key = "packing_allowed" if packed else "in_place"
        square = rate(4096, 4096, 4096, packed)
        shapes = {}
        for c in (2, 4, 8):
            for big, small in itertools.permutations(range(3), 2):
                d = [4096, 4096, 4096]
                d[big] *= c
                d[small] //= c
                shapes["%dx%dx%d" % tuple(d)] = round(rate(d[0], d[1], d[2], packed), 2)
        v = list(shapes.values())
        out[key] = {"square_4096": round(square, 2), "mean": round(statistics.mean(v), 2),
                    "std": round(statistics.pstdev(v), 2), "min": round(min(v), 2),
                    "std_over_mean": round(statistics.pstdev(v) / statistics.mean(v), 4),
                    "mean_over_square": round(statistics.mean(v) / square, 4), "shapes": shapes}
    out["paper_context"] = "AMULET with packing on one Xeon thread: std 2.9 % of the mean, mean within 1.7 % of square (Sec. 6.4)"
    print(json.dumps(out))
    return 0


def bench_workload(args, am, torch, np, wl) -> dict:
    """One named workload, measured as the header says: returns the JSON record."""
    spec, A, B, P = wl.make(args.workload)
    task, M, N, K = spec["task"], spec["M"], spec["N"], spec["K"]
    if task == "count_i8":
        return bench_count_i8(args, am, torch, np, spec, A, B)
    if spec.get("dtype") == "f64":
        return bench_f64(args, am, torch, np, wl, spec, A, B, P)
    tname = wl.TASK_NAMES[task]
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dP = torch.from_numpy(P).cuda() if P is not None else None
    dR = torch.zeros(M, N, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    if args.traffic_probe:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # 256 MiB read + 256 MiB written by one plain copy kernel
        torch.cuda.synchronize()
        if not args.no_tune:
            am.amulet_tune(task, M, N, K)
        for _ in range(args.steps):
            am.amulet_mmlike_f32(task, dA, dB, dP, dR)
        torch.cuda.synchronize()
        print("traffic probe done: 1 copy of %d bytes, %d launches of %s" %
              (src.numel() * 4, args.steps, am.amulet_shape_name(task, am.amulet_selected_shape(task, M, N, K))))
        return {}

    t0 = time.perf_counter()
    shape = am.amulet_selected_shape(task, M, N, K) if args.no_tune else am.amulet_tune(task, M, N, K)
    tune_s = time.perf_counter() - t0

    def time_library_sgemm():
        for _ in range(args.warmup):
            torch.mm(dA, dB)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            torch.mm(dA, dB)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    # the library SGEMM (rocBLAS / hipBLASLt behind torch.mm) on the same device buffers is timed
    # before and after our timed region and its faster run is the one compared against
    lib_before = time_library_sgemm() if tname == "identity" else None

    for _ in range(args.warmup):
        am.amulet_mmlike_f32(task, dA, dB, dP, dR)
    torch.cuda.synchronize()

    # per-launch HIP events on the stream the kernel runs on (torch's current stream)
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    with ShaderClock() as sclk:
        w0 = time.perf_counter()
        for i in range(args.steps):
            starts[i].record()
            am.amulet_mmlike_f32(task, dA, dB, dP, dR)
            stops[i].record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - w0) * 1e3
    sclk_mhz = sclk.median_mhz()
    kern_ms = [s.elapsed_time(e) for s, e in zip(starts, stops)]
    ms_per_step = wall_ms / args.steps
    kernel_ms_avg = sum(kern_ms) / len(kern_ms)
    kernel_ms_median = sorted(kern_ms)[len(kern_ms) // 2]

    flops = 2.0 * M * N * K
    value = flops / (ms_per_step * 1e-3) / 1e9                 # GFLOP/s, whole job
    achieved_tflops = flops / (kernel_ms_avg * 1e-3) / 1e12    # dominant (only) kernel
    ops = VALU_OPS_PER_PRODUCT[tname]
    ceiling_tflops = 2.0 * VALU_LANE_OPS_PER_S / ops / 1e12

    # parity spot check + CPU baseline: the oracle on a bounded sample of whole rows
    cpu = None
    parity = None
    if args.cpu_rows > 0:
        import oracle
        g = np.random.Generator(np.random.PCG64(99))
        rows = np.sort(g.choice(M, min(args.cpu_rows, M), replace=False))
        Rz = torch.zeros(M, N, dtype=torch.float32, device="cuda")
        am.amulet_mmlike_f32(task, dA, dB, dP, Rz)
        torch.cuda.synchronize()
        R_rows = Rz[torch.from_numpy(rows).cuda()].cpu().numpy()
        As = np.ascontiguousarray(A[rows])
        c0 = time.perf_counter()
        R_ref, ab, threads = oracle.mmlike_f32(task, As, B, P)
        cpu_s = time.perf_counter() - c0
        cpu = {"value": round(2.0 * len(rows) * N * K / cpu_s / 1e9, 3), "unit": "GFLOP/s (2MNK/t)",
               "cores": threads, "kind": "oracle",
               "sample": "%d whole rows of the %dx%dx%d workload (%.2e products), %.1f s"
                         % (len(rows), M, N, K, float(len(rows)) * N * K, cpu_s)}
        diff = np.abs(R_rows.astype(np.float64) - R_ref)
        # outputs whose terms are all zero must match exactly
        parity = float("inf") if np.any(diff[ab == 0] != 0) else float(np.max(diff / np.where(ab > 0, ab, 1.0)))

    # HBM bytes per launch measured with rocprofv3 --pmc (see profiles/), when recorded for this workload
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            rec = json.load(f).get(args.workload)
        if rec and rec.get("tile_shape") == am.amulet_shape_name(task, shape):   # measured for this very kernel
            traffic = rec["hbm_bytes_per_launch"]

    lib_ratio = None
    if tname == "identity":
        lib_ms = min(lib_before, time_library_sgemm())
        lib_ratio = {"library_sgemm_ms": round(lib_ms, 4), "ours_over_library_rate": round(lib_ms / kernel_ms_avg, 4)}

    # register-only issue rate of this task's instruction mix on this chip (measured ceiling)
    probe = None
    mix = {"identity": 0, "discount": 1, "boost": 2, "count_gt": 3}.get(tname)
    on_valu = am.amulet_shape_name(task, shape).startswith("valu")
    if mix is not None and on_valu and args.probe:
        pps = max(am.amulet_probe_valu(mix, w) for w in (4, 8))
        probe = {"mix": tname, "tflops_equiv": round(2.0 * pps / 1e12, 3),
                 "kernel_over_probe": round(achieved_tflops / (2.0 * pps / 1e12), 4)}

    # the stated targets: predicate tasks at >= 60 % of the fp32 vector peak at 8192^3 (above the
    # 25 % that four lane-operations per product allow: reported as missed, with the reason);
    # the identity task within 15 % of the library SGEMM
    target = None
    if tname == "identity" and lib_ratio is not None:
        target = {"what": "identity within 15 % of the library SGEMM", "met": bool(lib_ratio["ours_over_library_rate"] >= 0.85)}
    elif on_valu and tname != "identity":
        frac = achieved_tflops / FP32_VECTOR_PEAK_TFLOPS
        target = {"what": ">= 60 % of the fp32 vector peak", "met": bool(frac >= 0.60),
                  "note": "%g vector lane-operations per product cap the metric at %.1f %% of that peak"
                          % (ops, 100.0 / ops)}

    return {
        "metric": "effective GFLOP/s (2MNK/t), %s task %dx%dx%d fp32" % (tname, M, N, K),
        "value": round(value, 1),
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "task": tname, "M": M, "N": N, "K": K,
                   "tile_shape": am.amulet_shape_name(task, shape), "tuned": not args.no_tune,
                   "tune_seconds": round(tune_s, 3)},
        "pct_of_fp32_vector_peak": round(100.0 * value / 1e3 / FP32_VECTOR_PEAK_TFLOPS, 2),
        "roofline": {"bound": "alu" if on_valu else "mfma", "achieved": round(achieved_tflops, 3),
                     "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved_tflops / FP32_VECTOR_PEAK_TFLOPS, 4), "traffic": traffic,
                     "kernel_ms_avg": round(kernel_ms_avg, 4), "kernel_ms_median": round(kernel_ms_median, 4),
                     "valu_ops_per_product": ops,
                     "op_mix_ceiling_tflops": round(ceiling_tflops, 3),
                     "frac_of_op_mix_ceiling": round(achieved_tflops / ceiling_tflops, 4),
                     "shader_clock_mhz": sclk_mhz,
                     "frac_of_op_mix_ceiling_at_clock": None if not sclk_mhz else
                     round(achieved_tflops / (ceiling_tflops * sclk_mhz / 2400.0), 4)},
        "valu_probe": probe,
        "cpu_baseline": cpu,
        "parity_worst_ratio_on_sample": parity,
        "parity_ok": None if parity is None else bool(parity <= 1e-5),
        "target_met": target,
        "library_sgemm": lib_ratio,
        "paper_context": "AMULET Query 1 on one Xeon 6312U thread, double: SPR 7.50 = 15.0 GFLOP/s (Table 4)",
    }


# the other named workloads, measured after the headline's timed region in the default run
CONFIG_LEGS = ["cfg0_discount_256", "cfg1_boost_2048", "cfg2_identity_4096", "cfg3_count_i8_8192x8192x4096",
               "cfg4_discount_16384x2048x8192", "query3_count_gt_4096",
               "f64_discount_4096", "f64_boost_2048", "f64_identity_4096"]


def config_leg(name, args, am, torch, np, wl) -> dict:
    """A short run of one more named workload (3 warm-ups, 10 timed launches, the oracle on a
    small sample of whole rows): the figures a reader needs, without the headline's extras."""
    t0 = time.perf_counter()
    sub = argparse.Namespace(**vars(args))
    # enough untimed launches for about 0.1 s of work: the first launches after a pause run at other
    # clocks than a steady stream of them (a sub-millisecond kernel measures up to 10 % apart)
    ms_guess = {"cfg0_discount_256": 0.02, "cfg1_boost_2048": 0.6, "cfg2_identity_4096": 1.0,
                "cfg3_count_i8_8192x8192x4096": 0.25}.get(name, 5.0)
    sub.workload, sub.steps, sub.probe = name, max(10, min(args.steps, 20)), False
    # the legs run the built-in shape choices (the headline is the run that times amulet_tune): a
    # tune of a 0.2 ms kernel right after another workload has picked a shape that then ran 5 %
    # slower than the default, and a leg should measure the kernel, not that noise
    sub.no_tune = True
    sub.warmup = max(3, args.warmup, min(400, int(100.0 / ms_guess)))
    if wl.CONFIGS[name]["task"] == "count_i8":
        # (the matrix-core clock takes about a second of load to settle: 0.5 s of launches first, for
        # both forms of the join count alike)
        sub.warmup = max(sub.warmup, int(500.0 / ms_guess))
    M = wl.CONFIGS[name]["M"]
    sub.cpu_rows = min(M, 64) if wl.CONFIGS[name]["task"] != "count_i8" else 16   # count_i8 samples 4 x this
    rec = bench_workload(sub, am, torch, np, wl)
    roof = rec["roofline"]
    out = {"workload": name, "value": rec["value"], "unit": rec["unit"], "steps": sub.steps, "warmup": sub.warmup,
           "ms_per_step": rec["ms_per_step"], "kernel_ms_avg": roof["kernel_ms_avg"], "dtype": rec["dtype"],
           "tile_shape": rec["config"]["tile_shape"],
           "roofline": {k: roof[k] for k in ("bound", "achieved", "peak", "unit", "frac", "frac_of_op_mix_ceiling",
                                             "frac_of_mfma_probe", "shader_clock_mhz",
                                             "frac_of_op_mix_ceiling_at_clock", "assign_form") if k in roof},
           "parity_on_sample": rec.get("parity_worst_ratio_on_sample", rec.get("bit_exact_on_sample")),
           "parity_ok": rec["parity_ok"], "parity_sample": rec["cpu_baseline"]["sample"] if rec["cpu_baseline"] else None}
    for key in ("library_sgemm", "library_dgemm"):
        if rec.get(key):
            out[key] = rec[key]
    if rec.get("target_met"):
        out["target_met"] = rec["target_met"]
    out["seconds"] = round(time.perf_counter() - t0, 1)
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="headline_discount_8192")
    ap.add_argument("--no-tune", action="store_true", help="use the built-in default tile shape")
    ap.add_argument("--cpu-rows", type=int, default=512,
                    help="rows of the workload the CPU oracle is timed on (0 = skip); 512 rows of the "
                         "headline workload are about 13 s on 16 host threads")
    ap.add_argument("--no-configs", action="store_true",
                    help="default run only: leave out the short legs over the other named workloads "
                         "(the `configs` array of the JSON line)")
    ap.add_argument("--nonsquare", choices=["discount", "boost", "count_gt", "identity"], default=None,
                    help="instead of the workload: the paper's non-square protocol (18 shapes of equal work "
                         "around 4096^3) for this task, in place and with packing allowed")
    ap.add_argument("--i8-assign", action="store_true",
                    help="int8 join count: time (trace, count) the R = form, amulet_count_i8_assign, instead of R +=")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: one plain 256 MiB device copy (known HBM bytes, "
                         "the counter calibration) followed by --steps launches of the kernel; prints no JSON")
    args = ap.parse_args()
    args.probe = True
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); the path shards over rows of A "
              "without any exchange, but no multi-GPU run is part of it.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import amulet_workloads as wl
    import paper_2305_08872_amd as am

    am.load_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)

    if args.nonsquare:
        return bench_nonsquare(args, am, torch)
    out = bench_workload(args, am, torch, np, wl)
    if not out:
        return 0
    # The default run also puts every other named workload on record, each as a short leg of its
    # own after the headline's timed region (nothing of them runs inside it).
    if args.workload == "headline_discount_8192" and not args.no_configs:
        legs = []
        for name in CONFIG_LEGS:
            torch.cuda.empty_cache()
            legs.append(config_leg(name, args, am, torch, np, wl))
        out["configs"] = legs
        out["configs_seconds"] = round(sum(l["seconds"] for l in legs), 1)
    print(json.dumps(out))
    bad = [out["config"]["workload"]] if out.get("parity_ok") is False else []
    bad += [l["workload"] for l in out.get("configs", []) if l.get("parity_ok") is False]
    if bad:
        print("bench.py: sampled parity against the oracle FAILED for " + ", ".join(bad), file=sys.stderr)
        return 3
    return 0


if __name__ == "__main__":
    sys.exit(main())
