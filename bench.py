#!/usr/bin/env python3
"""Benchmark of the hot path: one "step" is one whole oz2_dgemm call (scaling,
residues, N INT8 GEMMs, CRT epilogue) on synthetic inputs resident in HBM.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--size 16384] [--moduli 16] [--phi 0.5]

Prints ONE JSON line on stdout: emulated FP64 TFLOP/s (2mnk / time) at
m = n = k = 16384, the roofline of the dominant kernel (the batched INT8 MFMA
GEMM, timed with HIP events on the call's stream inside the timed steps),
native FP64 GEMM on the same buffers, the accuracy of both against a
double-double product on sampled rows, the matrix cores' own rate and the board
power of both GEMMs, and the CPU oracle timed on a sub-block of the same problem.  Everything else goes to stderr.

    python bench.py --sweep NAME [--out FILE]

times other workloads, one JSON line per case into FILE: dgemm_4096, dgemm_16384, dgemm_16384_n14_15,
sgemm, nonsquare, modes (the benchmark configurations over their moduli counts), throughput_dgemm,
throughput_sgemm (m = n = k from 1024 to 16384, both modes), accuracy (error against N in the setting
of the paper's accuracy figure), general (transposed and prepared operands, bounded workspace), small
(launch-bound sizes, eager and as a graph), rank_k (short contractions), overlap (the overlapped form of a
call, an option, against the default single-stream form).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0          # MI355X dense INT8 MFMA, published
HBM_PEAK_GBS = 8000.0

def measured_gemm_traffic(dtype: str, size: int, num_moduli: int):
    """L2<->memory bytes per launch of k_int8_gemm for this workload, as measured with rocprofv3
    (FETCH_SIZE / WRITE_SIZE runs of this script, scaled by what the counters read for
    `--stage copy`).  The figure is not measured by this run: it is read from the committed
    summary under profiles/ that holds it, from a line of the form
        bench.roofline.traffic: dtype=f64 size=16384 N=16 launches=8 bytes=1.7e10 commit=abc1234
    (bytes per launch, the launches a call made in the profiled run, the commit the profile was
    taken at).  None when no summary covers the workload."""
    import glob
    import re
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        for line in open(path):
            if not line.startswith("bench.roofline.traffic:"):
                continue
            kv = dict(re.findall(r"(\w+)=(\S+)", line))
            if kv.get("dtype") == dtype and int(kv.get("size", -1)) == size and int(kv.get("N", -1)) == num_moduli:
                return {"bytes": float(kv["bytes"]), "launches": int(kv.get("launches", 1)), "commit": kv.get("commit"),
                        "file": os.path.basename(path)}
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class PowerSampler:
    """Samples the board power (and shader clock) that the amdgpu driver publishes in sysfs.

    A thread reads hwmon's power1_input (microwatts) and freq1_input (Hz) every few
    milliseconds; nothing of it touches the GPU.  `None` figures when the files are absent."""

    def __init__(self, torch, period_s: float = 0.005):
        import glob
        self.period = period_s
        self.power_file = self.freq_file = None
        cards = sorted(glob.glob("/sys/class/drm/card[0-9]*/device/hwmon/hwmon*/power1_input"))
        want = None
        try:
            want = "%02x:00" % torch.cuda.get_device_properties(0).pci_bus_id
        except Exception:
            pass
        for f in cards:
            dev = os.path.realpath(os.path.join(os.path.dirname(f), "..", ".."))
            if len(cards) == 1 or (want and want in os.path.basename(dev)):
                self.power_file = f
                fq = os.path.join(os.path.dirname(f), "freq1_input")
                self.freq_file = fq if os.path.exists(fq) else None
                break
        self.samples = []

    @staticmethod
    def _read(path):
        try:
            with open(path) as fh:
                return float(fh.read().strip())
        except (OSError, ValueError):
            return None

    def cap_watts(self):
        if not self.power_file:
            return None
        v = self._read(os.path.join(os.path.dirname(self.power_file), "power1_cap"))
        return v / 1e6 if v else None

    def run(self, torch, launch, seconds: float, settle_s: float):
        """Calls launch() back to back for about `seconds`; returns (calls per second, mean W,
        mean shader MHz) with the first `settle_s` of samples dropped."""
        import threading
        stop = threading.Event()
        samples = []

        def loop():
            while not stop.is_set():
                w = self._read(self.power_file) if self.power_file else None
                f = self._read(self.freq_file) if self.freq_file else None
                samples.append((time.perf_counter(), w, f))
                time.sleep(self.period)

        launch()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        launch()
        torch.cuda.synchronize()
        one = max(time.perf_counter() - t1, 1e-4)
        calls = max(3, int(seconds / one))
        th = threading.Thread(target=loop, daemon=True)
        th.start()
        t0 = time.perf_counter()
        for _ in range(calls):
            launch()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        stop.set()
        th.join()
        ws = [w for t, w, f in samples if w is not None and t - t0 >= settle_s]
        fs = [f for t, w, f in samples if f is not None and t - t0 >= settle_s]
        watts = sum(ws) / len(ws) / 1e6 if ws else None
        mhz = sum(fs) / len(fs) / 1e6 if fs else None
        return calls / elapsed, watts, mhz


def gemm_only(oz, torch, size, N, args) -> int:
    """Times oz2_int8_gemm alone on uniformly random int8 slices of the padded shape."""
    pad = lambda x, to: (x + to - 1) // to * to
    Mp = Np = pad(size, 256)
    Kp = pad(size, 128)
    g = torch.Generator(device="cuda").manual_seed(0)
    A = torch.randint(-128, 128, (N, Kp // 64, Mp, 64), dtype=torch.int8, device="cuda", generator=g)
    B = torch.randint(-128, 128, (N, Kp // 64, Np, 64), dtype=torch.int8, device="cuda", generator=g)
    C = torch.empty((N, Mp, Np), dtype=torch.int32, device="cuda")
    for _ in range(args.warmup):
        oz.oz2_int8_gemm(A, B, C, N, Mp, Np, Kp)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        oz.oz2_int8_gemm(A, B, C, N, Mp, Np, Kp)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    ops = 2.0 * Mp * Np * Kp * N
    tops = ops / (ms * 1e-3) / 1e12
    log(f"int8 gemm {N} x {Mp}x{Np}x{Kp}: {ms:.3f} ms, {tops:.0f} TOP/s ({100 * tops / INT8_PEAK_TOPS:.1f}% of peak)")
    print(json.dumps({"stage": "int8_gemm", "ms_per_launch": ms, "achieved_TOPs": tops,
                      "frac_of_int8_peak": tops / INT8_PEAK_TOPS, "batch": N, "Mp": Mp, "Np": Np,
                      "Kp": Kp, "steps": args.steps}), flush=True)
    return 0


def copy_only(torch, args) -> int:
    """A device-to-device copy of 4 GiB: reads 4 GiB and writes 4 GiB of HBM."""
    nbytes = 4 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(args.warmup):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    gbs = 2.0 * nbytes / (ms * 1e-3) / 1e9
    log(f"copy of {nbytes} B: {ms:.3f} ms, {gbs:.0f} GB/s read+write")
    print(json.dumps({"stage": "copy", "bytes_read": nbytes, "bytes_written": nbytes,
                      "ms_per_copy": ms, "GBps_read_plus_write": gbs, "steps": args.steps}),
          flush=True)
    return 0


SWEEPS = {
    # the parity-test configurations of the benchmark set, timed: (m, n, k, phi, fp64?, moduli)
    "dgemm_4096": [(4096, 4096, 4096, 0.5, True, list(range(12, 21)))],
    "dgemm_16384": [(16384, 16384, 16384, phi, True, [16, 17, 18, 19, 20]) for phi in (0.5, 1.0, 2.0)],
    # the moduli counts at which the paper quotes its DGEMM-level results (Section 5.2)
    "dgemm_16384_n14_15": [(16384, 16384, 16384, 0.5, True, [14, 15])],
    "sgemm": [(8192, 8192, 8192, 0.5, False, [5, 6, 7, 8, 9]),
              (16384, 16384, 16384, 0.5, False, [5, 6, 7, 8, 9])],
    "nonsquare": [(8192, 8192, 65536, 1.0, True, [18])],
    # fast against accurate mode on inputs with a wide exponent range
    "modes": [(8192, 8192, 8192, phi, True, [14, 15, 16, 17, 18]) for phi in (0.5, 2.0, 4.0)],
    # throughput against the matrix size, both modes, at the moduli counts of Section 5.2
    # (the setting of the paper's DGEMM and SGEMM throughput and time-breakdown figures)
    "throughput_dgemm": [(s, s, s, 0.5, True, [14, 15, 16, 17]) for s in (1024, 2048, 4096, 8192, 16384)],
    "throughput_sgemm": [(s, s, s, 0.5, False, [6, 7, 8]) for s in (1024, 2048, 4096, 8192, 16384)],
}
BOTH_MODES = ("modes", "throughput_dgemm", "throughput_sgemm")


def sweep(oz, torch, name, args) -> int:
    """Times oz2_dgemm / oz2_sgemm over the moduli counts of a configuration and measures the
    error of each result (and of the native GEMM) against a double-double product on three
    sampled rows.  One JSON line per (shape, phi, N) goes to the file named by --out."""
    import numpy as np
    import synth_inputs as S
    from oracle import oz2_oracle as O              # reference leg only
    path = args.out or f"sweep_{name}.jsonl"
    if os.path.dirname(path):
        os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        for (m, n, k, phi, is_double, moduli) in SWEEPS[name]:
            np_dt, t_dt = (np.float64, torch.float64) if is_double else (np.float32, torch.float32)
            A, B = S.gemm_inputs(m, n, k, phi, seed=0, dtype=np_dt)
            dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
            dC = torch.empty((m, n), dtype=t_dt, device="cuda")
            rows = np.array([0, m // 3, m - 1])
            trows = torch.from_numpy(rows).cuda()
            hi, lo, ab = O.dd_rows(A.astype(np.float64), B.astype(np.float64), rows)
            err = lambda c: float(np.max(np.abs((c.astype(np.float64) - hi) - lo) / ab))
            torch.mm(dA, dB, out=dC)
            torch.cuda.synchronize()
            native_reps = max(3, min(200, int(2e11 / (2.0 * m * n * k))))
            t1 = time.perf_counter()
            for _ in range(native_reps):
                torch.mm(dA, dB, out=dC)
            torch.cuda.synchronize()
            native_tflops = 2.0 * m * n * k / ((time.perf_counter() - t1) / native_reps) / 1e12
            native_err = err(dC[trows].cpu().numpy())
            modes = [False, True] if name in BOTH_MODES else [args.accurate]
            for N, accurate in [(N, a) for N in moduli for a in modes]:
                if accurate:
                    fn = oz.oz2_dgemm_accurate if is_double else oz.oz2_sgemm_accurate
                else:
                    fn = oz.oz2_dgemm if is_double else oz.oz2_sgemm
                for _ in range(args.warmup):
                    fn(m, n, k, 1.0, dA, k, dB, n, 0.0, dC, n, N)
                torch.cuda.synchronize()
                # the calls back to back (small sizes: enough of them to time), then per-stage
                # times from profiled calls, which wait for their events one by one
                reps = max(args.steps, min(200, int(2e11 / (2.0 * m * n * k))))
                t0 = time.perf_counter()
                for _ in range(reps):
                    fn(m, n, k, 1.0, dA, k, dB, n, 0.0, dC, n, N)
                torch.cuda.synchronize()
                dt = (time.perf_counter() - t0) / reps
                oz.oz2_set_profiling(True)
                stage_ms = np.zeros(4)
                for _ in range(args.steps):
                    fn(m, n, k, 1.0, dA, k, dB, n, 0.0, dC, n, N)
                    stage_ms += np.array(oz.oz2_last_stage_times_ms())
                oz.oz2_set_profiling(False)
                rec = {"m": m, "n": n, "k": k, "phi": phi, "dtype": "f64" if is_double else "f32",
                       "mode": "accurate" if accurate else "fast", "num_moduli": N, "ms": 1e3 * dt, "emulated_tflops": 2.0 * m * n * k / dt / 1e12,
                       "stage_ms": (stage_ms / args.steps).round(3).tolist(),
                       "err_emulated": err(dC[trows].cpu().numpy()), "native_tflops": native_tflops,
                       "err_native": native_err}
                log(json.dumps(rec))
                f.write(json.dumps(rec) + "\n")
                f.flush()
            del dA, dB, dC
    print(json.dumps({"sweep": name, "file": path}), flush=True)
    oz.oz2_release()
    return 0


def sweep_general(oz, torch, args) -> int:
    """Times the general entry points on one shape (--size, --moduli, FP64): the four
    transposition cases of oz2_dgemm_op, a product of prepared operands (and the
    preparation itself), and products cut into panels by a workspace limit.  Every result is
    compared with the plain call's bit for bit.  One JSON line per case goes to --out."""
    import numpy as np
    import synth_inputs as S
    m = n = k = args.size
    N = args.moduli
    path = args.out or "sweep_general.jsonl"
    if os.path.dirname(path):
        os.makedirs(os.path.dirname(path), exist_ok=True)
    A, B = S.gemm_inputs(m, n, k, args.phi, seed=0)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dAt, dBt = dA.t().contiguous(), dB.t().contiguous()
    want = oz.matmul(dA, dB, N).clone()
    dC = torch.empty_like(want)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        oz.oz2_set_profiling(True)
        stage_ms = np.zeros(4)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
            stage_ms += np.array(oz.oz2_last_stage_times_ms())
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        oz.oz2_set_profiling(False)
        return dt, (stage_ms / args.steps).round(3).tolist()

    with open(path, "w") as f:
        def emit(case, dt, stage_ms, **extra):
            rec = {"case": case, "m": m, "n": n, "k": k, "num_moduli": N, "ms": 1e3 * dt,
                   "emulated_tflops": 2.0 * m * n * k / dt / 1e12, "stage_ms": stage_ms,
                   "equals_plain_call": bool(torch.equal(dC, want))}
            rec.update(extra)
            log(json.dumps(rec))
            f.write(json.dumps(rec) + "\n")
            f.flush()

        for opA, opB, X, Y in ((0, 0, dA, dB), (0, 1, dA, dBt), (1, 0, dAt, dB), (1, 1, dAt, dBt)):
            dC.zero_()
            dt, st = timed(lambda: oz.oz2_dgemm_op(opA, opB, 0, m, n, k, 1.0, X, X.shape[1], Y, Y.shape[1],
                                                   0.0, dC, n, N))
            emit(f"op(A)={'NT'[opA]} op(B)={'NT'[opB]}", dt, st)

        # prepared operands: Algorithm 1 lines 1-5 once per matrix, then products only
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        L = oz.oz2_prepare_d(0, 0, m, k, dA, k, N)
        R = oz.oz2_prepare_d(1, 0, n, k, dB, n, N)
        torch.cuda.synchronize()
        prep_ms = 1e3 * (time.perf_counter() - t0)
        dC.zero_()
        dt, st = timed(lambda: oz.oz2_dgemm_prepared(L, R, 1.0, 0.0, dC, n))
        emit("prepared operands (product only)", dt, st, prepare_both_ms_incl_alloc=prep_ms,
             operand_bytes=[L.nbytes, R.nbytes])
        L.free(); R.free()

        # bounded workspace: C in 4 and in 16 panels
        least = oz.oz2_workspace_min_bytes(m, n, k, N)
        for frac in (4, 16):
            if m // 256 < frac:
                continue
            limit = least - N * 256 * 256 + N * (m * n // frac)
            oz.oz2_set_workspace_limit(limit)
            oz.oz2_release()
            dC.zero_()
            dt, st = timed(lambda: oz.oz2_dgemm(m, n, k, 1.0, dA, k, dB, n, 0.0, dC, n, N))
            emit(f"workspace limited to 1/{frac} of the products", dt, st,
                 panels=list(oz.oz2_last_panels()), workspace_bytes=limit)
        oz.oz2_set_workspace_limit(0)
    print(json.dumps({"sweep": "general", "file": path}), flush=True)
    oz.oz2_release()
    return 0


def sweep_small(oz, torch, args) -> int:
    """Launch-bound sizes: one oz2_dgemm call is four dependent kernel launches at these sizes
    (nine from 4096^3 on), so the call is timed eagerly and as a replayed HIP graph, next to the
    native GEMM."""
    import numpy as np
    import synth_inputs as S
    N = args.moduli
    path = args.out or "sweep_small.jsonl"
    if os.path.dirname(path):
        os.makedirs(os.path.dirname(path), exist_ok=True)

    def per_call(fn, reps):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    with open(path, "w") as f:
        for size in (256, 512, 1024, 2048, 4096):
            m = n = k = size
            A, B = S.gemm_inputs(m, n, k, args.phi, seed=0)
            dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
            dC = torch.empty((m, n), dtype=torch.float64, device="cuda")
            call = lambda: oz.oz2_dgemm(m, n, k, 1.0, dA, k, dB, n, 0.0, dC, n, N)
            reps = 200 if size <= 1024 else 50
            eager = per_call(call, reps)
            want = dC.clone()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                call()
            dC.zero_()
            graph = per_call(g.replay, reps)
            same = bool(torch.equal(dC, want))
            native = per_call(lambda: torch.mm(dA, dB, out=dC), reps)
            rec = {"m": m, "n": n, "k": k, "num_moduli": N, "eager_us": 1e6 * eager, "graph_us": 1e6 * graph,
                   "native_us": 1e6 * native, "graph_equals_eager": same,
                   "emulated_tflops_graph": 2.0 * m * n * k / graph / 1e12,
                   "native_tflops": 2.0 * m * n * k / native / 1e12}
            log(json.dumps(rec))
            f.write(json.dumps(rec) + "\n")
            del g
    print(json.dumps({"sweep": "small", "file": path}), flush=True)
    oz.oz2_release()
    return 0


def sweep_accuracy(oz, torch, args) -> int:
    """The setting of the paper's accuracy figure (Section 5.1): m = n = 1024, k = 1024 and 16384,
    several phi, fast and accurate mode over the number of moduli, FP64 and FP32; the error
    of each result and of the native GEMM against a double-double product on 16 sampled rows.
    One JSON line per (type, k, phi) with the error per mode and N goes to --out."""
    import numpy as np
    import synth_inputs as S
    from oracle import oz2_oracle as O              # reference leg only
    path = args.out or "sweep_accuracy.jsonl"
    if os.path.dirname(path):
        os.makedirs(os.path.dirname(path), exist_ok=True)
    m = n = 1024
    rows = np.arange(0, m, m // 16)
    with open(path, "w") as f:
        for is_double, moduli in ((True, list(range(8, 21))), (False, list(range(2, 13)))):
            np_dt, t_dt = (np.float64, torch.float64) if is_double else (np.float32, torch.float32)
            for k in (1024, 16384):
                for phi in (0.5, 1.0, 1.5, 2.0, 4.0):
                    A, B = S.gemm_inputs(m, n, k, phi, seed=0, dtype=np_dt)
                    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
                    trows = torch.from_numpy(rows).cuda()
                    hi, lo, ab = O.dd_rows(A.astype(np.float64), B.astype(np.float64), rows)
                    err = lambda c: float(np.max(np.abs((c.astype(np.float64) - hi) - lo) / ab))
                    # second measure: the error relative to the entry itself, |c - AB| / |AB|
                    ref_abs = np.abs(hi + lo)
                    rel = lambda c: float(np.max(np.abs((c.astype(np.float64) - hi) - lo)
                                                 / np.where(ref_abs == 0, 1.0, ref_abs)))
                    native = torch.mm(dA, dB)[trows].cpu().numpy()
                    rec = {"dtype": "f64" if is_double else "f32", "m": m, "n": n, "k": k, "phi": phi,
                           "measure": "max |c - dd(AB)| / (|A||B|) on 16 rows",
                           "measure_rel": "max |c - dd(AB)| / |dd(AB)| on the same rows",
                           "native": err(native), "fast": {}, "accurate": {},
                           "native_rel": rel(native), "fast_rel": {}, "accurate_rel": {}}
                    for N in moduli:
                        for accurate in (False, True):
                            c = oz.matmul(dA, dB, N, accurate=accurate)[trows].cpu().numpy()
                            rec["accurate" if accurate else "fast"][str(N)] = err(c)
                            rec["accurate_rel" if accurate else "fast_rel"][str(N)] = rel(c)
                    log(json.dumps(rec))
                    f.write(json.dumps(rec) + "\n")
    print(json.dumps({"sweep": "accuracy", "file": path}), flush=True)
    oz.oz2_release()
    return 0


def sweep_rank_k(oz, torch, args) -> int:
    """Short contractions, the shape of a blocked factorisation's trailing update (the use the
    paper names for N = 14, 15): C <- C - A B with m = n large and k = 512 ... 4096, against the
    native GEMM doing the same update.  One JSON line per shape goes to --out."""
    import numpy as np
    import synth_inputs as S
    N = args.moduli if args.moduli != 16 else 15
    path = args.out or "sweep_rank_k.jsonl"
    if os.path.dirname(path):
        os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        for (m, n, k) in ((16384, 16384, 512), (16384, 16384, 1024), (16384, 16384, 2048),
                          (16384, 16384, 4096), (32768, 32768, 1024)):
            A, B = S.gemm_inputs(m, n, k, args.phi, seed=0)
            dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
            dC = torch.zeros((m, n), dtype=torch.float64, device="cuda")
            call = lambda: oz.oz2_dgemm(m, n, k, -1.0, dA, k, dB, n, 1.0, dC, n, N)
            for _ in range(args.warmup):
                call()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                call()
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / args.steps
            oz.oz2_set_profiling(True)
            stage_ms = np.zeros(4)
            for _ in range(args.steps):
                call()
                stage_ms += np.array(oz.oz2_last_stage_times_ms())
            oz.oz2_set_profiling(False)
            dC.addmm_(dA, dB, beta=1.0, alpha=-1.0)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(3):
                dC.addmm_(dA, dB, beta=1.0, alpha=-1.0)
            torch.cuda.synchronize()
            nat = (time.perf_counter() - t1) / 3
            rec = {"m": m, "n": n, "k": k, "num_moduli": N, "alpha": -1.0, "beta": 1.0, "ms": 1e3 * dt,
                   "emulated_tflops": 2.0 * m * n * k / dt / 1e12,
                   "stage_ms": (stage_ms / args.steps).round(3).tolist(), "native_ms": 1e3 * nat,
                   "native_tflops": 2.0 * m * n * k / nat / 1e12}
            log(json.dumps(rec))
            f.write(json.dumps(rec) + "\n")
            del dA, dB, dC
    print(json.dumps({"sweep": "rank_k", "file": path}), flush=True)
    oz.oz2_release()
    return 0


def sweep_overlap(oz, torch, args) -> int:
    """The overlapped form of a call (an option: conversion of later panels on a second stream
    where the rule allows it) against the default single-stream form, on the same device and
    buffers, in turns.  One JSON line per workload goes to --out."""
    import numpy as np
    import synth_inputs as S
    path = args.out or "sweep_overlap.jsonl"
    if os.path.dirname(path):
        os.makedirs(os.path.dirname(path), exist_ok=True)
    cases = [(16384, 16384, 16384, 16, True, False), (16384, 16384, 16384, 16, True, True),
             (16384, 16384, 16384, 8, False, False), (8192, 8192, 65536, 18, True, False),
             (8192, 8192, 8192, 16, True, False), (16384, 16384, 4096, 15, True, False)]
    with open(path, "w") as f:
        for (m, n, k, N, is_double, accurate) in cases:
            A, B = S.gemm_inputs(m, n, k, args.phi, seed=0, dtype=np.float64 if is_double else np.float32)
            dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
            dC = torch.empty((m, n), dtype=dA.dtype, device="cuda")
            call = lambda: oz.matmul(dA, dB, N, out=dC, accurate=accurate)
            ms = {False: [], True: []}
            try:
                for _ in range(2):                         # in turns, so that drift hits both alike
                    for on in (False, True):
                        oz.oz2_set_overlap(on)
                        for _ in range(args.warmup):
                            call()
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                        for _ in range(args.steps):
                            call()
                        torch.cuda.synchronize()
                        ms[on].append(1e3 * (time.perf_counter() - t0) / args.steps)
                panels = list(oz.oz2_last_panels())            # of the overlapped form
            finally:
                oz.oz2_set_overlap(False)
            rec = {"m": m, "n": n, "k": k, "num_moduli": N, "dtype": "f64" if is_double else "f32",
                   "mode": "accurate" if accurate else "fast", "single_stream_ms": min(ms[False]),
                   "overlapped_ms": min(ms[True]), "panels_of_the_overlapped_form": panels}
            log(json.dumps(rec))
            f.write(json.dumps(rec) + "\n")
            del dA, dB, dC
    print(json.dumps({"sweep": "overlap", "file": path}), flush=True)
    oz.oz2_release()
    return 0


def sweep_launches(oz, torch, args) -> int:
    """One INT8 GEMM launch per product (option OZ2_OPT_CUT_LAUNCHES off) against the default, in
    which the launches of a large product are cut into parts of C and K ranges, on the same device
    and buffers, in turns; the results must be the same bits.  One JSON line per workload goes to
    --out."""
    import numpy as np
    import synth_inputs as S
    from paper_2508_03984_amd import binding as b
    path = args.out or "sweep_launches.jsonl"
    if os.path.dirname(path):
        os.makedirs(os.path.dirname(path), exist_ok=True)
    cases = [(16384, 16384, 16384, 16, True, False), (16384, 16384, 16384, 14, True, False),
             (16384, 16384, 16384, 16, True, True), (16384, 16384, 16384, 8, False, False),
             (8192, 8192, 65536, 18, True, False), (10000, 9000, 20000, 15, True, False),
             (8192, 8192, 8192, 16, True, False), (16384, 16384, 4096, 15, True, False)]
    with open(path, "w") as f:
        for (m, n, k, N, is_double, accurate) in cases:
            A, B = S.gemm_inputs(m, n, k, args.phi, seed=0, dtype=np.float64 if is_double else np.float32)
            dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
            del A, B
            dC = torch.empty((m, n), dtype=dA.dtype, device="cuda")
            call = lambda: oz.matmul(dA, dB, N, out=dC, accurate=accurate)
            ms, launches, sums = {False: [], True: []}, {}, {}
            try:
                for _ in range(2):                         # in turns, so that drift hits both alike
                    for on in (False, True):
                        oz.oz2_ctx_set_option(None, b.OZ2_OPT_CUT_LAUNCHES, on)
                        for _ in range(args.warmup):
                            call()
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                        for _ in range(args.steps):
                            call()
                        torch.cuda.synchronize()
                        ms[on].append(1e3 * (time.perf_counter() - t0) / args.steps)
                        launches[on] = oz.oz2_last_gemm_launches()
                        if on not in sums:
                            sums[on] = dC.clone()
                same = bool(torch.equal(sums[False], sums[True]))
            finally:
                oz.oz2_ctx_set_option(None, b.OZ2_OPT_CUT_LAUNCHES, True)
            rec = {"m": m, "n": n, "k": k, "num_moduli": N, "dtype": "f64" if is_double else "f32",
                   "mode": "accurate" if accurate else "fast", "one_launch_ms": min(ms[False]),
                   "cut_launches_ms": min(ms[True]), "launches": [launches[False], launches[True]],
                   "same_bits": same}
            log(json.dumps(rec))
            f.write(json.dumps(rec) + "\n")
            del dA, dB, dC, sums
    print(json.dumps({"sweep": "launches", "file": path}), flush=True)
    oz.oz2_release()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--size", type=int, default=16384, help="m = n = k")
    ap.add_argument("--moduli", type=int, default=16)
    ap.add_argument("--phi", type=float, default=0.5)
    ap.add_argument("--sgemm", action="store_true", help="FP32 emulation (oz2_sgemm)")
    ap.add_argument("--accurate", action="store_true",
                    help="accurate mode of Section 4.2 (oz2_dgemm_accurate / oz2_sgemm_accurate)")
    ap.add_argument("--int32-products", action="store_true",
                    help="diagnostic pipeline: the GEMM stores int32 sums, the epilogue reduces them")
    ap.add_argument("--inputs", choices=["synthetic", "ones"], default="synthetic",
                    help="ones: A = B = 1 everywhere, so every residue slice is one constant (diagnostic: "
                         "the matrix cores then draw little power and the chip does not lower its clock)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the MFMA-only probe, the library INT8 GEMM and the power legs")
    ap.add_argument("--stage", choices=["all", "int8_gemm", "copy"], default="all",
                    help="int8_gemm: time only the batched INT8 GEMM on random residues; "
                         "copy: a plain 4 GiB device copy (calibrates the profiler's HBM byte "
                         "counters); both print a reduced JSON line")
    ap.add_argument("--sweep", choices=sorted(SWEEPS) + ["general", "small", "accuracy", "rank_k", "overlap", "launches"], default=None,
                    help="time a whole configuration of the benchmark set over its moduli counts; "
                         "one JSON line per case goes to --out")
    ap.add_argument("--out", default=None, help="file for --sweep (default: sweep_<name>.jsonl)")
    ap.add_argument("--cpu-block", type=int, default=1536,
                    help="the oracle is timed on C[0:b, 0:b] with the full k")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
            "(no collectives, sharding or rank code exist here)")
        return 2

    import numpy as np
    import torch

    import paper_2508_03984_amd as oz
    import synth_inputs as S

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 2
    torch.cuda.set_device(0)
    oz.load()                                        # raises if liboz2.so is missing
    oz.oz2_set_int32_products(args.int32_products)

    m = n = k = args.size
    N = args.moduli
    if args.sweep == "general":
        return sweep_general(oz, torch, args)
    if args.sweep == "small":
        return sweep_small(oz, torch, args)
    if args.sweep == "accuracy":
        return sweep_accuracy(oz, torch, args)
    if args.sweep == "rank_k":
        return sweep_rank_k(oz, torch, args)
    if args.sweep == "overlap":
        return sweep_overlap(oz, torch, args)
    if args.sweep == "launches":
        return sweep_launches(oz, torch, args)
    if args.sweep:
        return sweep(oz, torch, args.sweep, args)
    if args.stage == "int8_gemm":
        return gemm_only(oz, torch, m, N, args)
    if args.stage == "copy":
        return copy_only(torch, args)
    np_dt, t_dt = (np.float32, torch.float32) if args.sgemm else (np.float64, torch.float64)
    log(f"generating inputs {m}x{k}, {k}x{n} phi={args.phi} ...")
    t0 = time.time()
    if args.inputs == "ones":
        A, B = np.ones((m, k), np_dt), np.ones((k, n), np_dt)
    else:
        A, B = S.gemm_inputs(m, n, k, args.phi, seed=0, dtype=np_dt)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dC = torch.empty((m, n), dtype=t_dt, device="cuda")
    log(f"  done in {time.time() - t0:.1f}s")
    if args.accurate:
        fn = oz.oz2_sgemm_accurate if args.sgemm else oz.oz2_dgemm_accurate
    else:
        fn = oz.oz2_sgemm if args.sgemm else oz.oz2_dgemm
    stream = torch.cuda.current_stream()

    def step():
        fn(m, n, k, 1.0, dA, k, dB, n, 0.0, dC, n, N, stream)

    oz.oz2_set_profiling(True)                      # HIP events around the four stages
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    stage_ms = np.zeros(4)
    t_start = time.perf_counter()
    for _ in range(args.steps):
        step()
        stage_ms += np.array(oz.oz2_last_stage_times_ms())   # waits for this step's last event
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    oz.oz2_set_profiling(False)
    stage_ms /= args.steps
    ms_per_step = 1e3 * elapsed / args.steps
    tflops = 2.0 * m * n * k / (elapsed / args.steps) / 1e12
    panel_rows, panel_cols, panels = oz.oz2_last_panels()
    gemm_launches = oz.oz2_last_gemm_launches()                  # of the last step: per launch panel and K range of 2^17
    log(f"oz2 {'sgemm' if args.sgemm else 'dgemm'} N={N}: {ms_per_step:.2f} ms/step, "
        f"{tflops:.1f} emulated TFLOP/s; stages [shift, residues, gemm, epilogue] ms = "
        f"{np.round(stage_ms, 3).tolist()}; {panels} panel(s) of {panel_rows} x {panel_cols}, "
        f"{gemm_launches} INT8 GEMM launch(es)")
    # dominant kernel: the batched INT8 GEMM on the padded slices
    pad = lambda x, to: (x + to - 1) // to * to
    Mp, Np, Kp = pad(m, 256), pad(n, 256), pad(k, 128)
    gemm_ops = 2.0 * Mp * Np * Kp * N
    gemm_tops = gemm_ops / (stage_ms[2] * 1e-3) / 1e12            # stage_ms[2]: all GEMM launches of a step
    E = 4 if args.sgemm else 8
    PB = 4 if args.int32_products else 1                        # bytes per product entry
    stage_bytes = [
        E * (m * k + 2 * k * n) + 4 * (m + n),                  # shifts: A once, B twice (max, then sum)
        E * (m * k + k * n) + N * (Mp * Kp + Np * Kp),          # residues
        N * (Mp * Kp + Np * Kp) + PB * N * Mp * Np,             # GEMM compulsory traffic
        PB * N * m * n + E * m * n,                             # epilogue
    ]
    stage_gbs = [b / (t * 1e-3) / 1e9 if t > 0 else 0.0 for b, t in zip(stage_bytes, stage_ms)]

    # what a plain device copy moves on this device (read + write), as the practical ceiling of
    # the bandwidth-bound stages: dC <- dA, 2 GiB each way at the default size
    copy_gbs = None
    if dA.numel() == dC.numel():
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        dC.copy_(dA)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(3):
            dC.copy_(dA)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 2.0 * dA.numel() * dA.element_size() / (e0.elapsed_time(e1) / 3 * 1e-3) / 1e9

    # native GEMM on the same buffers (rocBLAS / hipBLASLt through torch)
    torch.mm(dA, dB, out=dC)
    torch.cuda.synchronize()
    reps = 3
    t1 = time.perf_counter()
    for _ in range(reps):
        torch.mm(dA, dB, out=dC)
    torch.cuda.synchronize()
    native_tflops = 2.0 * m * n * k / ((time.perf_counter() - t1) / reps) / 1e12
    log(f"native {'SGEMM' if args.sgemm else 'DGEMM'}: {native_tflops:.1f} TFLOP/s")

    # the matrix cores alone, the library's INT8 GEMM, and board power (Section 5.3 of the paper
    # reports power efficiency; here: sysfs board power while each GEMM runs back to back)
    device = power = None
    if not args.no_extras:
        const_tops, cus, mhz = oz.oz2_mfma_probe(False, 0.25)
        rand_tops, _, _ = oz.oz2_mfma_probe(True, 0.25)
        device = {"name": torch.cuda.get_device_name(0), "compute_units": cus, "nominal_clock_mhz": mhz,
                  "mfma_only_TOPs": {"constant_operands": const_tops, "random_operands": rand_tops},
                  "int8_gemm_frac_of_mfma_only_random": gemm_tops / rand_tops}
        try:
            g = torch.Generator(device="cuda").manual_seed(0)
            ia = torch.randint(-128, 128, (Mp, Kp), dtype=torch.int8, device="cuda", generator=g)
            ib = torch.randint(-128, 128, (Np, Kp), dtype=torch.int8, device="cuda", generator=g).t()
            torch._int_mm(ia, ib)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(N):                                # as many slices as one launch of ours
                torch._int_mm(ia, ib)
            e1.record()
            torch.cuda.synchronize()
            device["library_int8_gemm_TOPs"] = gemm_ops / (e0.elapsed_time(e1) * 1e-3) / 1e12
            del ia, ib
        except Exception as ex:                               # not every build of torch has it
            device["library_int8_gemm_TOPs"] = None
            log(f"torch._int_mm not usable: {ex!r}"[:200])
        log(f"device {device}")
        ps = PowerSampler(torch)
        if ps.power_file:
            cps_e, w_e, f_e = ps.run(torch, step, 2.5, 1.0)
            cps_n, w_n, f_n = ps.run(torch, lambda: torch.mm(dA, dB, out=dC), 2.5, 1.0)
            gf = 2.0 * m * n * k / 1e9
            power = {"source": "amdgpu hwmon power1_input / freq1_input, mean over 1.5 s of back-to-back calls",
                     "cap_W": ps.cap_watts(),
                     "emulated": {"W": w_e, "shader_MHz": f_e, "GFLOPS_per_W": gf * cps_e / w_e if w_e else None},
                     "native": {"W": w_n, "shader_MHz": f_n, "GFLOPS_per_W": gf * cps_n / w_n if w_n else None}}
            log(f"power {power}")

    # accuracy of both on a few sampled rows against a double-double product (CPU)
    from oracle import oz2_oracle as O              # allowed here: baseline / reference leg only
    rows = np.unique(np.concatenate([[0, m - 1], (np.arange(14) + 1) * (m // 15) + np.arange(14) * 37 % max(m // 15, 1)]) % m)
    native_rows = dC[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    step()
    torch.cuda.synchronize()
    emu_rows = dC[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    A64, B64 = (A.astype(np.float64), B.astype(np.float64)) if args.sgemm else (A, B)
    hi, lo, ab = O.dd_rows(A64, B64, rows)
    err = lambda c: float(np.max(np.abs((c - hi) - lo) / ab))
    accuracy = {"measure": f"max |c - dd(AB)| / (|A||B|) on {len(rows)} sampled rows",
                "emulated": err(emu_rows), "native": err(native_rows)}
    log(f"accuracy {accuracy}")

    cpu = None
    if not args.no_cpu_baseline:
        b = min(args.cpu_block, m)
        As, Bs = np.ascontiguousarray(A[:b, :]), np.ascontiguousarray(B[:, :b])
        t2 = time.perf_counter()
        ref = O.gemm(As, Bs, N, is_double=not args.sgemm, accurate=args.accurate)
        dt = time.perf_counter() - t2
        cpu = {"value": 2.0 * b * b * k / dt / 1e12, "unit": "TFLOP/s", "cores": O.num_threads(),
               "kind": "oracle",
               "sample": f"C[0:{b},0:{b}] of the same problem (full k={k}, N={N}), all of Algorithm 1; "
                         f"{dt:.1f} s"}
        sub = dC[:b, :b].cpu().numpy().astype(np.float64)
        r = ref["C"].astype(np.float64)
        # shifts of B's columns and A's rows do not depend on the other rows/columns, so the
        # sub-block of the full GPU result must equal the oracle's result on the sub-problem
        if not args.accurate:                   # accurate-mode shifts depend on all of A and B
            cpu["gpu_vs_oracle_max_rel_diff"] = float(
                np.max(np.abs(sub - r) / np.where(r == 0, 1.0, np.abs(r))))
        log(f"cpu oracle {cpu}")

    traffic = measured_gemm_traffic("f32" if args.sgemm else "f64", m, N) if m == n == k else None
    out = {
        "metric": "emulated FP64 TFLOPS (2mnk/s) at m=n=k=16384; INT8 MFMA % of peak"
                  if not args.sgemm else "emulated FP32 TFLOPS (2mnk/s); INT8 MFMA % of peak",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "int8",
        "dtype_note": "INT8 MFMA products with exact INT32 accumulation; scaling, residues and CRT "
                      "reconstruction in FP64; inputs and output " + ("FP32" if args.sgemm else "FP64"),
        "data": "synthetic" if args.inputs == "synthetic" else "all ones (diagnostic run, not the benchmark)",
        "config": {"workload": f"{'SGEMM' if args.sgemm else 'DGEMM'} emulation m=n=k={m}, "
                               f"{'fp32' if args.sgemm else 'fp64'} row-major, phi={args.phi}, "
                               f"seed 0/1, {'accurate' if args.accurate else 'fast'} mode, N={N} moduli, "
                               f"alpha=1 beta=0",
                   "num_moduli": N, "m": m, "n": n, "k": k, "phi": args.phi},
        "roofline": {"bound": "mfma", "kernel": "k_int8_gemm (batched over moduli)",
                     "achieved": gemm_tops, "peak": INT8_PEAK_TOPS, "unit": "TFLOP/s",
                     "frac": gemm_tops / INT8_PEAK_TOPS,
                     # per launch of THIS run (the profiled run's bytes per call over this run's launches)
                     "traffic": traffic["bytes"] * traffic["launches"] / gemm_launches if traffic else None,
                     "traffic_source": traffic,
                     "ops_per_launch": gemm_ops / gemm_launches,
                     "avg_launch_ms": float(stage_ms[2] / gemm_launches),
                     "launches_per_step": gemm_launches,
                     "note": "INT8 multiply-adds counted as 2 ops each, against the dense INT8 peak"},
        "stages": {"ms": {"shifts": float(stage_ms[0]), "residues": float(stage_ms[1]),
                          "int8_gemm": float(stage_ms[2]), "epilogue": float(stage_ms[3])},
                   "hbm_GBps_algorithmic": {"shifts": stage_gbs[0], "residues": stage_gbs[1],
                                            "int8_gemm": stage_gbs[2], "epilogue": stage_gbs[3]},
                   "hbm_peak_GBps": HBM_PEAK_GBS, "device_copy_GBps_read_plus_write": copy_gbs},
        "native_gemm_tflops": native_tflops,
        "speedup_vs_native": tflops / native_tflops,
        "accuracy": accuracy,
        "device": device,
        "power": power,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    oz.oz2_release()
    return 0


if __name__ == "__main__":
    sys.exit(main())
