#!/usr/bin/env python3
"""Benchmark of the fused lazy-array path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload normalize] [--no-extras]

One step = one pass of the whole hot path over one batch of synthetic input:
wrap the device buffers as leaves, record the NumPy-style program, partition,
look the kernels up in the cache, launch, mark materialised, release.  The
headline workload is the 8192x8192 broadcast normalisation; inputs are resident
in HBM before the timed region and three buffer sets are rotated so that the
256 MB Infinity Cache cannot serve repeats.  Prints ONE JSON line.

Metric: effective GB/s = (unique input bytes + output bytes) / time.

Timing: HIP events on the stream the kernels are launched on (the context uses
torch's current stream).  The K timed steps of a region run back to back; events
recorded inside the region at (up to) ten block boundaries give a per-step median
and minimum over blocks beside the average of the whole region, without
lengthening it.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP32_MFMA_PEAK_TFLOPS = 157.3
VALU_PEAK_TLANEOPS = 256 * 64 * 2.4e9 / 1e12   # vector instructions x lanes per second: 256 compute units, 64 lanes each, 2.4 GHz
BLACKSCHOLES_VALU_PER_ELEMENT = 124            # SQ_INSTS_VALU per wave / 1024 elements per wave (profiles/gr_map_blackscholes_pmc.txt)
ARGNAMES = {"gemm": ("A", "B"), "cumsum_axis0": ("X",), "cumsum": ("x",), "blackscholes": ("S", "K", "T"), "chain": ("a", "b"), "normalize": ("X", "mu", "sigma", "gamma", "beta"), "softmax": ("X",),
            "stencil": ("I",), "logreg": ("X", "w", "y")}
# kernel whose launches dominate each workload
DOMINANT = {"gemm": "gr_gemm", "cumsum_axis0": "gr_scan", "cumsum": "gr_scan", "blackscholes": "gr_map", "chain": "gr_map", "normalize": "gr_map", "softmax": "gr_rowred", "stencil": "gr_map", "logreg": "gr_gemv_pair"}


def out_shape(name, p):
    return {"gemm": lambda: (p["m"], p["n"]), "chain": lambda: (p["n"],), "cumsum": lambda: (p["n"],), "cumsum_axis0": lambda: (p["rows"], p["cols"]), "blackscholes": lambda: (p["n"],), "normalize": lambda: (p["rows"], p["cols"]), "softmax": lambda: (p["rows"], p["cols"]),
            "stencil": lambda: (p["rows"] - 4, p["cols"] - 4), "logreg": lambda: (p["cols"],)}[name]()


def algorithmic_bytes_per_launch(name, p):
    """Bytes one launch of the dominant kernel has to move: every distinct input element once plus the output."""
    from paper_1901_03771_amd import workloads as wl
    if name == "logreg":  # one pass over X for both contractions; the residual r is written once on the way
        return wl.unique_bytes(name, **p) + 4 * p["rows"]
    return wl.unique_bytes(name, **p)


class Workload:
    """Device-resident buffer sets of one configuration and the step that evaluates it."""

    def __init__(self, name, ctx, nsets, size=None):
        import torch
        from paper_1901_03771_amd import lazy as gr, workloads as wl
        self.name, self.ctx, self.gr, self.wl, self.torch = name, ctx, gr, wl, torch
        self.p = dict(wl.FULL[name])
        if size:
            self.p.update(size)
        self.sets = []
        for s in range(nsets):
            arrays = wl.make_inputs(name, salt=s, **self.p)
            dev = {k: torch.from_numpy(v).cuda() for k, v in arrays.items()}
            out = torch.empty(out_shape(name, self.p), dtype=torch.float32, device="cuda")
            self.sets.append((dev, out))
        self.i = 0
        self.unique_bytes = wl.unique_bytes(name, **self.p)
        self.program = None

    def step(self):
        dev, out = self.sets[self.i % len(self.sets)]
        self.i += 1
        leaves = {k: self.ctx.array(t) for k, t in dev.items()}
        self.wl.PROGRAMS[self.name](self.gr, **leaves).materialize_into(out)
        return out

    def record(self):
        """Records the request once for replay (gr_program_create) with every input rebindable."""
        dev, _ = self.sets[0]
        leaves = {k: self.ctx.array(t) for k, t in dev.items()}
        self.program = self.ctx.program(self.wl.PROGRAMS[self.name](self.gr, **leaves), [leaves[k] for k in ARGNAMES[self.name]])
        self.order = [[dev_[k] for k in ARGNAMES[self.name]] for dev_, _ in self.sets]

    def replay(self):
        k = self.i % len(self.sets)
        self.i += 1
        self.program.run(self.order[k], self.sets[k][1])


def time_region(torch, step, steps, warmup, blocks=10):
    """`warmup` untimed steps, then exactly `steps` steps back to back between two events; events at block
    boundaries inside the region give per-step times per block.  Returns (region ms, wall ms, [us per step per block])."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    nb = max(1, min(blocks, steps))
    bounds = [steps * b // nb for b in range(nb + 1)]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(nb + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for b in range(nb):
        for _ in range(bounds[b + 1] - bounds[b]):
            step()
        ev[b + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    per_block = [ev[b].elapsed_time(ev[b + 1]) / (bounds[b + 1] - bounds[b]) * 1e3 for b in range(nb)]
    return max(ev[0].elapsed_time(ev[nb]), 0.0), wall_ms, per_block


def spin_up(torch, step, min_ms=40.0, min_steps=20):
    """Untimed steps for at least `min_ms` of device time: drawing a configuration's inputs on the host leaves the GPU
    idle for about a second, and for some 25 ms after that launches run up to 10 % slower than in steady state."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    done, n = 0.0, min_steps
    while done < min_ms:
        e0.record()
        for _ in range(n):
            step()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        done += ms
        n = max(min_steps, min(4000, int(n * (min_ms - done) / max(ms, 1e-3)) + 1))


def median(xs):
    s = sorted(xs)
    return s[len(s) // 2] if len(s) % 2 else 0.5 * (s[len(s) // 2 - 1] + s[len(s) // 2])


def hbm_roofline(kernel, alg_bytes, avg_us, per_block_us, launches, **more):
    achieved = alg_bytes / (avg_us * 1e-6) / 1e9
    r = {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": round(achieved / HBM_PEAK_GBS, 4), "launches": launches, "avg_launch_us": round(avg_us, 2),
         "median_us": round(median(per_block_us), 2), "min_us": round(min(per_block_us), 2),
         "algorithmic_bytes_per_launch": alg_bytes}
    r.update(more)
    return r


def cpu_baseline(name, target_cpu_s=20.0):
    """The oracle as it stands, timed on the host cores on a bounded sample of the workload: on every core the
    process may use (`value`, `cores`) and on one thread (`single_thread`), about `target_cpu_s` core-seconds in
    all; eager NumPy on the same sample as context (the paper's own denominator, Section 4.2)."""
    import numpy as np
    import oracle as ora
    from paper_1901_03771_amd import workloads as wl
    cores = len(os.sched_getaffinity(0))
    full = wl.FULL[name]

    def run(sz, threads):
        ora.set_threads(threads)
        arrays = wl.make_inputs(name, **sz)
        t0 = time.perf_counter()
        wl.PROGRAMS[name](ora, **{k: ora.array(v) for k, v in arrays.items()}).numpy()
        return time.perf_counter() - t0, arrays

    def leg(threads, budget_core_s):
        if name in ("chain", "blackscholes", "cumsum"):
            size = dict(n=full["n"])
        elif name == "gemm":
            size = dict(m=128, k=full["k"], n=full["n"])
        else:
            size = dict(rows=64 if name != "logreg" else 4096, cols=full["cols"])
        t, arrays = run(size, threads)
        if "rows" in size:  # scale the row count towards the budget, capped at the full workload
            rows = int(min(full["rows"], max(size["rows"], size["rows"] * (budget_core_s / threads / 3) / max(t, 1e-3))))
            size = dict(rows=rows, cols=full["cols"])
        times = []
        while not times or (sum(times) * threads < budget_core_s and len(times) < 20):
            t, arrays = run(size, threads)
            times.append(t)
        t = median(times)
        nbytes = wl.unique_bytes(name, **size)
        return {"value": round(nbytes / t / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
                "sample": f"{name} program on " + ", ".join(f"{k}={v}" for k, v in size.items()) +
                          f" (same recipe, seed and column count as the timed workload), median of {len(times)} runs, "
                          f"{t:.2f} s wall each on {threads} OpenMP thread{'s' if threads > 1 else ''}, {sum(times) * threads:.0f} core-seconds in all"}, arrays, nbytes

    out, arrays, nbytes = leg(cores, 0.7 * target_cpu_s)
    out["host_cores_available"] = cores
    if cores > 1:
        single, _, _ = leg(1, 0.3 * target_cpu_s)
        out["single_thread"] = single
    if name != "blackscholes":  # NumPy has no erf
        t0 = time.perf_counter()
        wl.PROGRAMS[name](np, **arrays)
        out["numpy_eager_GBps_context"] = round(nbytes / (time.perf_counter() - t0) / 1e9, 3)
    return out


def traffic_from_profiles(name):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this kernel and workload (not measured in
    this run: counters need a profiler pass of their own)."""
    rel = os.path.join("profiles", f"{DOMINANT[name]}_{name}_pmc.txt")
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1]), rel
    except OSError:
        pass
    return None, None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)   # ~10 ms: the GPU idles while the inputs are drawn on the host, then takes a while to run at full speed
    ap.add_argument("--workload", default="normalize", choices=sorted(ARGNAMES))
    ap.add_argument("--sets", type=int, default=3)
    ap.add_argument("--no-extras", action="store_true", help="skip the supplementary configurations and ceilings")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--calibrate", type=int, default=0, metavar="N",
                    help="also launch the plain copy kernel N times on the workload's first array (reference for rocprofv3 counters)")
    ap.add_argument("--no-launch-events", action="store_true", help="skip the instrumented cross-check pass (one HIP event pair per launch)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path would shard by rows, one context per GPU); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1901_03771_amd import lazy as gr, workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    ctx = gr.Context(device=0)

    name = args.workload
    w = Workload(name, ctx, args.sets)
    t0 = time.perf_counter()
    w.step()
    torch.cuda.synchronize()
    # first request of a structure the process has never seen: record, plan, generate; while hipRTC
    # compiles on a host thread the request itself is served by the byte-code interpreter
    cold_ms = (time.perf_counter() - t0) * 1e3
    cold_interpreted = ctx.stats()["interp_launches"] > 0
    t0 = time.perf_counter()
    ctx.compile_wait()
    compile_wait_ms = (time.perf_counter() - t0) * 1e3
    ctx.set_option("interp", 0)  # everything timed below runs the generated kernels

    # Timed region: exactly K steps back to back after W untimed ones.  No per-launch instrumentation here.
    dev_ms, wall_ms, per_block = time_region(torch, w.step, args.steps, args.warmup)
    ms_per_step = dev_ms / args.steps
    value = w.unique_bytes / (ms_per_step * 1e-3) / 1e9

    # Roofline of the dominant kernel.  Its average launch duration over the timed region is
    # region time / launches (kernels run back to back, so this includes the launch gaps and is
    # an upper bound); a second, instrumented pass brackets every launch with its own event
    # pair as a cross-check against the rocprofv3 kernel trace.
    traffic, traffic_src = traffic_from_profiles(name)
    roofline = hbm_roofline(DOMINANT[name], algorithmic_bytes_per_launch(name, w.p), ms_per_step * 1e3, per_block, args.steps,
                            traffic=traffic, traffic_source=(traffic_src + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by the plain copy kernel; committed summary, not measured in this run)") if traffic_src else None)
    if name == "gemm":  # a dense contraction: priced against the matrix cores, not against HBM
        flops = 2 * w.p["m"] * w.p["k"] * w.p["n"]
        tf = flops / (ms_per_step * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": "gr_gemm", "achieved": round(tf, 1), "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tf / FP32_MFMA_PEAK_TFLOPS, 4), "launches": args.steps, "avg_launch_us": round(ms_per_step * 1e3, 1),
                    "median_us": round(median(per_block), 1), "min_us": round(min(per_block), 1), "algorithmic_flops_per_launch": flops, "traffic": None}
    if not args.no_launch_events:
        ctx.set_option("profile", 1)
        ctx.profile_reset()
        time_region(torch, w.step, min(args.steps, 100), 5)
        n, total_ms = ctx.profile_read(DOMINANT[name])
        ctx.set_option("profile", 0)
        roofline["per_launch_event_us"] = round(total_ms / max(n, 1) * 1e3, 2)

    result = {
        "metric": "effective GB/s of fused DAG eval (unique in+out bytes) and % of MI355X HBM peak",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{name}: " + ", ".join(f"{k}={v}" for k, v in w.p.items()), "buffer_sets": args.sets,
                   "unique_bytes_per_step": w.unique_bytes},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "us_per_step_median_of_blocks": round(median(per_block), 2), "us_per_step_min_of_blocks": round(min(per_block), 2),
        "host_wall_ms_per_step": round(wall_ms / args.steps, 5),
        "cold_first_call_ms": round(cold_ms, 2), "cold_first_call_interpreted": cold_interpreted,
        "compile_wait_after_first_call_ms": round(compile_wait_ms, 2),
        "roofline": roofline,
    }

    if args.calibrate:
        src, dst = w.sets[0][0][ARGNAMES[name][0]], w.sets[1][0][ARGNAMES[name][0]]
        for _ in range(args.calibrate):
            ctx.stream_copy(dst, src)
        torch.cuda.synchronize()

    if not args.no_extras:
        extras, rooflines = {}, {}
        # practical ceiling of the box: plain copy and read-only kernels, rotating over the same
        # buffer sets as the workload so that the Infinity Cache cannot serve the reads
        first = ARGNAMES[name][0]
        pairs = [(s_[0][first].reshape(-1), s_[1].reshape(-1)) for s_ in w.sets]
        nel = min(min(a.numel(), b.numel()) for a, b in pairs) // 4 * 4
        if nel >= (1 << 22):
            pairs = [(a[:nel], b[:nel]) for a, b in pairs]
            sink = torch.zeros(4096, device="cuda")
            k = [0]

            def copy_step():
                k[0] += 1
                ctx.stream_copy(pairs[k[0] % len(pairs)][1], pairs[k[0] % len(pairs)][0])

            def read_step():
                k[0] += 1
                ctx.stream_read(pairs[k[0] % len(pairs)][0], sink)
            for label, fn, nbytes in (("stream_copy", copy_step, 8 * nel), ("stream_read", read_step, 4 * nel)):
                d_ms, _, blocks = time_region(torch, fn, 100, 20)
                extras[label + "_GBps"] = round(nbytes / (d_ms / 100 * 1e-3) / 1e9, 1)
                rooflines[label] = hbm_roofline("gr_" + label + "_kernel", nbytes, d_ms / 100 * 1e3, blocks, 100)
        del w
        torch.cuda.empty_cache()

        # the other configurations (and two scaled pointwise chains): each spun up to steady state first
        others = [("chain", None), ("chain", dict(n=1 << 27)), ("blackscholes", dict(n=1 << 26)), ("softmax", None), ("stencil", None), ("logreg", None), ("normalize", None)]
        for oname, size in others:
            if oname == name and size is None:
                continue
            ow = Workload(oname, ctx, 3 if size is None else 2, size)
            small = oname == "chain" and size is None
            k = 2000 if small else 100
            spin_up(torch, ow.step)
            d_ms, o_wall, blocks = time_region(torch, ow.step, k, 0)
            label = oname if size is None else f"{oname}_n2^{size['n'].bit_length() - 1}"
            us = d_ms / k * 1e3
            extras[label + "_GBps"] = round(ow.unique_bytes / (us * 1e-6) / 1e9, 1)
            extras[label + "_us_per_step"] = round(us, 2)
            rooflines[label] = hbm_roofline(DOMINANT[oname], algorithmic_bytes_per_launch(oname, ow.p), us, blocks, k,
                                            **({"note": "12 MiB working set: resident in L2 / Infinity Cache, bound by launch rate and host work per step, not by HBM"} if small else {}),
                                            **({"note": "ALU-bound: log, exp, sqrt, two erf and four divisions per element"} if oname == "blackscholes" else {}))
            if oname == "blackscholes":
                # Vector-ALU roofline: one vector instruction per lane and cycle on each of the 64 lanes of a compute
                # unit (256 CUs at 2.4 GHz; packed FP32 is not used), against the 124 vector instructions per element
                # that rocprofv3 counts for this kernel (profiles/gr_map_blackscholes_pmc.txt: SQ_INSTS_VALU per wave / 1024)
                ops = BLACKSCHOLES_VALU_PER_ELEMENT * ow.p["n"] / (us * 1e-6) / 1e12
                rooflines[label + "_alu"] = {"bound": "alu", "kernel": "gr_map", "achieved": round(ops, 2), "peak": VALU_PEAK_TLANEOPS, "unit": "T lane-instructions/s",
                                             "frac": round(ops / VALU_PEAK_TLANEOPS, 4), "valu_instructions_per_element": BLACKSCHOLES_VALU_PER_ELEMENT,
                                             "note": "instruction count from the committed counter profile, time measured here; seven of the instructions per element are transcendental"}
            if small:
                # the same request recorded once and replayed (gr_program_run): launches only
                extras[label + "_host_wall_us_per_step"] = round(o_wall / k * 1e3, 2)
                ow.record()
                spin_up(torch, ow.replay)
                d_ms, o_wall, blocks = time_region(torch, ow.replay, k, 0)
                us = d_ms / k * 1e3
                extras[label + "_replay_GBps"] = round(ow.unique_bytes / (us * 1e-6) / 1e9, 1)
                extras[label + "_replay_us_per_step"] = round(us, 2)
                extras[label + "_replay_host_wall_us_per_step"] = round(o_wall / k * 1e3, 2)
                rooflines[label + "_replay"] = hbm_roofline("gr_map", algorithmic_bytes_per_launch(oname, ow.p), us, blocks, k,
                                                            note="recorded once, replayed: launches only; 12 MiB working set, cache-resident")
                ow.program.close()
            del ow
            torch.cuda.empty_cache()
        # the same GPU without fusion: one kernel per recorded op, every intermediate through HBM
        # (the eager model the paper starts from, Section 1)
        uctx = gr.Context(device=0)
        uctx.set_option("fusion", 0)
        uctx.set_option("interp", 0)
        for oname in ("normalize", "softmax"):
            ow = Workload(oname, uctx, 2)
            d_ms, _, _ = time_region(torch, ow.step, 20, 3)
            extras[oname + "_unfused_GBps"] = round(ow.unique_bytes / (d_ms / 20 * 1e-3) / 1e9, 1)
            del ow
            torch.cuda.empty_cache()
        uctx.close()
        # the byte-code interpreter that answers a request while its kernel is still being compiled
        ictx = gr.Context(device=0)
        ictx.set_option("interp", 2)
        for oname in ("normalize", "stencil", "softmax"):
            ow = Workload(oname, ictx, 2)
            d_ms, _, _ = time_region(torch, ow.step, 10, 2)
            extras[oname + "_interpreted_GBps"] = round(ow.unique_bytes / (d_ms / 10 * 1e-3) / 1e9, 1)
            del ow
            torch.cuda.empty_cache()
        ictx.close()
        # first request for a row-resident reduction in a context that has never seen it (and may not read
        # the on-disk cache): the interpreter's row kernel answers while hipRTC compiles
        cctx = gr.Context(device=0)
        cctx.set_option("disk_cache", 0)
        ow = Workload("softmax", cctx, 2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ow.step()
        torch.cuda.synchronize()
        extras["softmax_cold_first_call_ms"] = round((time.perf_counter() - t0) * 1e3, 2)
        extras["softmax_cold_first_call_interpreted"] = cctx.stats()["interp_launches"] > 0
        t0 = time.perf_counter()
        cctx.compile_wait()
        extras["softmax_compile_wait_after_first_call_ms"] = round((time.perf_counter() - t0) * 1e3, 2)
        del ow
        torch.cuda.empty_cache()
        cctx.close()

        # rows beyond the five configurations: two-stage reduction, map-scan, matrix product, the full Jacobi loop
        def timed(fn, iters, spin_ms=40.0):
            spin_up(torch, fn, min_ms=spin_ms, min_steps=2)
            d_ms, _, blocks = time_region(torch, fn, iters, 0)
            return d_ms / iters, blocks

        n = 1 << 27
        xs = [torch.rand(n, device="cuda") for _ in range(2)]
        out1 = torch.empty((), device="cuda")
        k = [0]

        def red():
            k[0] += 1
            gr.sum(gr.sqrt(ctx.array(xs[k[0] % 2]))).materialize_into(out1)
        ms, blocks = timed(red, 40)
        extras["sum_sqrt_n2^27_GBps"] = round(4 * n / (ms * 1e-3) / 1e9, 1)
        rooflines["sum_sqrt_n2^27"] = hbm_roofline("gr_reduce", 4 * n, ms * 1e3, blocks, 40)
        outn = torch.empty(n, device="cuda")

        def scan():
            k[0] += 1
            gr.cumsum(ctx.array(xs[k[0] % 2]), 0).materialize_into(outn)
        ms, blocks = timed(scan, 20)
        extras["cumsum_n2^27_GBps"] = round(8 * n / (ms * 1e-3) / 1e9, 1)
        extras["cumsum_n2^27_us"] = round(ms * 1e3, 1)
        rooflines["cumsum_n2^27"] = hbm_roofline("gr_scan", 8 * n, ms * 1e3, blocks, 20)
        del xs, outn
        torch.cuda.empty_cache()
        m2 = [torch.rand(8192, 8192, device="cuda") for _ in range(3)]
        outm = [torch.empty(8192, 8192, device="cuda") for _ in range(3)]   # rotated like the workloads' buffer sets

        def colscan():
            k[0] += 1
            gr.cumsum(ctx.array(m2[k[0] % 3]), 0).materialize_into(outm[k[0] % 3])
        ms, blocks = timed(colscan, 20)
        extras["cumsum_axis0_8192_GBps"] = round(8 * 8192 * 8192 / (ms * 1e-3) / 1e9, 1)
        extras["cumsum_axis0_8192_us"] = round(ms * 1e3, 1)
        rooflines["cumsum_axis0_8192"] = hbm_roofline("gr_scan", 8 * 8192 * 8192, ms * 1e3, blocks, 20)
        del m2, outm
        torch.cuda.empty_cache()
        ga, gb = torch.randn(4096, 4096, device="cuda"), torch.randn(4096, 4096, device="cuda")
        gc = torch.empty(4096, 4096, device="cuda")
        ms, blocks = timed(lambda: (ctx.array(ga) @ ctx.array(gb)).materialize_into(gc), 40, spin_ms=250.0)   # (matrix-core clocks settle slowly: the first 100 ms ran 3-6 % slower)
        tf = 2 * 4096 ** 3 / (ms * 1e-3) / 1e12
        extras["gemm_4096_f32_TFLOPs"] = round(tf, 1)
        rooflines["gemm_4096_f32"] = {"bound": "mfma", "kernel": "gr_gemm", "achieved": round(tf, 1), "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                                      "frac": round(tf / FP32_MFMA_PEAK_TFLOPS, 4), "launches": 40, "avg_launch_us": round(ms * 1e3, 1),
                                      "median_us": round(median(blocks), 1), "min_us": round(min(blocks), 1), "algorithmic_flops_per_launch": 2 * 4096 ** 3}
        del ga, gb, gc
        jac_bytes = 4 * 8192 * 8192 + 4 * 8190 * 8190
        sweeps = 10
        for label, owned in (("jacobi_8192", False), ("jacobi_lent_8192", None), ("jacobi_owned_8192", True)):
            # wrapped: the caller's tensor is the grid's storage (stencil -> temporary -> copy back); lent: the caller
            # lends a second tensor and the sweeps alternate between the two; owned: the library's own copy (each
            # sweep writes a second buffer, copies the border once and swaps)
            if owned is None:
                grid = ctx.array(torch.rand(8192, 8192, device="cuda"), second=torch.empty(8192, 8192, device="cuda"))
            else:
                grid = ctx.array(torch.rand(8192, 8192, device="cuda"))
            if owned:
                grid = grid.copy()
            ms, blocks = timed(lambda: wl.jacobi(gr, grid, sweeps), 10)
            extras[label + "_GBps_per_sweep"] = round(jac_bytes / (ms / sweeps * 1e-3) / 1e9, 1)
            extras[label + "_us_per_sweep"] = round(ms / sweeps * 1e3, 1)
            rooflines[label] = hbm_roofline("gr_map", jac_bytes, ms / sweeps * 1e3, [b / sweeps for b in blocks], 10 * sweeps)
            del grid
            torch.cuda.empty_cache()
        result["supplementary"] = extras
        result["supplementary_rooflines"] = rooflines

    result["stats"] = {k: (round(v, 2) if isinstance(v, float) else v) for k, v in ctx.stats().items()}
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(name)
    ctx.close()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
