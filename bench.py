#!/usr/bin/env python3
"""Benchmark of the segmented-operation hot path on one MI355X.

Default run (the contract line): the headline workload, the segmented
inclusive scan of n = 2^28 int8 values into int32 with segment lengths uniform
in [1, 4096] and bit-packed flags.  One "step" is one mmv_segscan call on
inputs that already sit in HBM: workspace reset kernel + the single-pass scan
kernel.  Prints ONE JSON line with the whole-job throughput (G elements/s), the
HBM roofline of the scan kernel measured with HIP events inside the timed
region (on every fourth step: an event pair costs about 5 us of stream time),
and the CPU oracle timed on the host beside it.

`--report FILE` additionally times all five workloads, both variants (matrix
cores / shuffle-only ablation) and the streaming-copy reference with the same
read:write mix, and writes the table as JSON lines to FILE.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth


class HipEvents:
    """hipEvent_t handles through the HIP runtime that torch has loaded."""

    def __init__(self):
        import torch
        path = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
        self.hip = ctypes.CDLL(path if os.path.exists(path) else "libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.made = []

    def create(self) -> int:
        ev = ctypes.c_void_p()
        if self.hip.hipEventCreate(ctypes.byref(ev)) != 0:
            raise RuntimeError("hipEventCreate failed")
        self.made.append(ev)
        return ev.value

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = ctypes.c_float()
        if self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return float(ms.value)

    def destroy_all(self):
        for ev in self.made:
            self.hip.hipEventDestroy(ev)
        self.made = []


EVENTS_EVERY = 1
LAST_KERNEL_SAMPLES: list = []   # kernel times of the last time_steps() call that used events


def time_steps(step, steps: int, warmup: int, events: HipEvents | None):
    """Runs warmup + steps calls of step(); returns (wall ms per step, mean kernel ms or None)."""
    import torch
    from paper_2506_23906_amd import binding as B
    for _ in range(warmup):
        step()
    pairs = [(events.create(), events.create()) for _ in range(0, steps, EVENTS_EVERY)] if events else []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        if events:
            if k % EVENTS_EVERY == 0:
                B.mmv_set_kernel_events(*pairs[k // EVENTS_EVERY])
            else:
                B.mmv_set_kernel_events(None, None)
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kernel_ms = None
    if events:
        B.mmv_set_kernel_events(None, None)
        samples = [events.elapsed_ms(a, b) for a, b in pairs]
        kernel_ms = float(np.mean(samples))
        LAST_KERNEL_SAMPLES[:] = samples
        events.destroy_all()
    return (t1 - t0) * 1e3 / steps, kernel_ms


def load_traffic(name: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload (counters cannot be read
    from inside this process), and a label that says so; (None, reason) if there is no such summary."""
    rel = os.path.join("profiles", name + "_hbm_traffic.txt")
    path = os.path.join(ROOT, rel)
    if os.path.exists(path):
        with open(path) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch"):
                    return int(line.split("=")[1]), ("replayed from %s (two rocprofv3 --pmc runs of this command, FETCH_SIZE "
                                                     "and WRITE_SIZE scaled by a copy of known size); not measured in this run" % rel)
    return None, "no counter summary for this workload under profiles/"


def oracle_baseline(x, f, repeats: int = 3):
    """The sequential CPU oracle, as it stands, on the same workload (one thread); returns (best seconds, result)."""
    import oracle
    best, ref = None, None
    for _ in range(repeats):
        t0 = time.perf_counter()
        ref = oracle.segscan(x, f)
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    return best, ref


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--log2n", type=int, default=28, help="vector length of the headline workload")
    ap.add_argument("--variant", default="mfma", choices=["mfma", "shuffle"])
    ap.add_argument("--input-copies", type=int, default=3,
                    help="the steps rotate over this many copies of the inputs (3 x 288 MiB is more than the "
                         "256 MiB memory-side cache, so no step finds its inputs cached from an earlier one)")
    ap.add_argument("--events-every", type=int, default=4,
                    help="record the kernel events on every n-th timed step only (an event pair costs about "
                         "5 us of stream time, which would otherwise be charged to every step)")
    ap.add_argument("--density", type=float, default=None,
                    help="uniformly random flags of this density instead of the segment lengths of the workload "
                         "(for profiling; changes config.workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--report", default=None, help="also time every workload and write JSON lines here")
    ap.add_argument("--copy-only", action="store_true",
                    help="run only the streaming copy reference (1 GiB in, 1 GiB out), for counter calibration")
    ap.add_argument("--copy-mix", default="1024:1024", metavar="IN:OUT",
                    help="with --copy-only: MiB read and MiB written per launch (256:1024 = the scan's 1:4 mix, "
                         "1024:0 = read only, 0:1024 = write only)")
    ap.add_argument("--segsum-only", type=float, default=None, metavar="DENSITY",
                    help="run only mmv_segsum on the int8 values with uniformly random flags of this density "
                         "(--steps calls, --variant), for counter runs; prints the kernel time")
    ap.add_argument("--lib", default=None,
                    help="load this build of libmmvseg.so instead of the one in the package (e.g. one made by "
                         "paper_2506_23906_amd.build.build(extra=['-DMMV_CHUNK_SUM=0'], out=...), to compare tunables)")
    args = ap.parse_args()
    global EVENTS_EVERY
    EVENTS_EVERY = max(1, args.events_every)
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path would shard by contiguous ranges with one "
              "exchange of per-GPU carries; that is design only); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import torch
    from paper_2506_23906_amd import binding as B
    from paper_2506_23906_amd import workloads as W
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if args.lib:
        B.LIB_PATH = os.path.abspath(args.lib)
    B.load()
    if args.segsum_only is not None:
        n = 1 << args.log2n
        x, _ = W.segscan_i8_uniform_len(n)
        f = W.uniform_density_flags(n, args.segsum_only, 78)
        xt = torch.from_numpy(x).cuda()
        ft = torch.from_numpy(W.pack_flags(f).view(np.int32)).cuda()
        out = torch.empty(int(f.sum()) + 16, dtype=torch.int32, device="cuda")
        nseg = torch.empty(1, dtype=torch.int64, device="cuda")
        ws = B.new_workspace(B.MMV_OP_SEGSUM, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
        EVENTS_EVERY = 1
        ms, kernel_ms = time_steps(lambda: B.mmv_segsum(xt, ft, n=n, out=out, nseg=nseg, variant=args.variant, ws=ws),
                                   args.steps, args.warmup, HipEvents())
        assert B.mmv_workspace_status(ws) == 0
        nbytes = n + n // 8 + int(f.sum()) * 4
        print(json.dumps({"segsum_only": True, "n": n, "density": args.segsum_only, "variant": args.variant,
                          "segments": int(f.sum()), "kernel_ms": kernel_ms, "ms_per_call": ms, "algo_bytes": nbytes,
                          "gb_s_kernel": nbytes / kernel_ms / 1e6, "frac_of_peak_kernel": nbytes / kernel_ms / 1e6 / HBM_PEAK_GBS}))
        return 0
    if args.copy_only:
        in_bytes, out_bytes = (int(v) << 20 for v in args.copy_mix.split(":"))
        src = torch.zeros(max(in_bytes, 16), dtype=torch.uint8, device="cuda")
        dst = torch.empty(max(out_bytes, 16), dtype=torch.uint8, device="cuda")
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        B.mmv_stream_copy(src, dst, in_bytes, out_bytes)
        a.record()
        for _ in range(args.steps):
            B.mmv_stream_copy(src, dst, in_bytes, out_bytes)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / args.steps
        print(json.dumps({"copy_only": True, "in_bytes": in_bytes, "out_bytes": out_bytes, "launches": args.steps + 1,
                          "ms_per_launch": ms, "gb_s": (in_bytes + out_bytes) / ms / 1e6}))
        return 0
    events = HipEvents()

    n = 1 << args.log2n
    x, f = W.segscan_i8_uniform_len(n)
    if args.density is not None:
        f = W.uniform_density_flags(n, args.density, 77)
    xt = torch.from_numpy(x).cuda()
    ft = torch.from_numpy(W.pack_flags(f).view(np.int32)).cuda()
    copies = [(xt, ft)] + [(xt.clone(), ft.clone()) for _ in range(max(1, args.input_copies) - 1)]
    zt = torch.empty(n, dtype=torch.int32, device="cuda")
    ws = B.new_workspace(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
    turn = [0]

    def step():
        xk, fk = copies[turn[0] % len(copies)]
        turn[0] += 1
        B.mmv_segscan(xk, fk, n=n, z=zt, variant=args.variant, ws=ws)

    ms_per_step, kernel_ms = time_steps(step, args.steps, args.warmup, events)
    assert B.mmv_workspace_status(ws) == 0
    algo_bytes = n * (1 + 4) + ((n + 31) // 32) * 4          # values in, result out, packed flags in
    achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9
    line = {
        "metric": "segmented-scan G elem/s + achieved HBM GB/s (%% of peak), n=2^%d" % args.log2n,
        "value": n / (ms_per_step * 1e-3) / 1e9,
        "unit": "Gelem/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "i32",
        "data": "synthetic",
        "config": {
            "workload": "segscan_i8_uniform_len: segmented inclusive scan, n=2^%d int8 in [-8,8] -> int32, "
                        "%s, bit-packed flags, seed %d"
                        % (args.log2n, "segment lengths U{1..4096}" if args.density is None
                           else "uniformly random flags of density %g" % args.density, W.SEEDS["segscan_i8_uniform_len"]),
            "variant": args.variant,
            "input_copies_rotated": len(copies),
            "kernel_events_every_nth_step": EVENTS_EVERY,
            "tile_elems": B.mmv_tile_elems(),
            "kernel_ms": kernel_ms,
            "kernel_ms_median": float(np.median(LAST_KERNEL_SAMPLES)),
            "kernel_ms_min": float(np.min(LAST_KERNEL_SAMPLES)),
            "workspace_reset_kernel_in_ms_per_step": True,   # the events of kernel_ms bracket the scan kernel alone
            "hbm_frac_of_peak_whole_step": algo_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": None,
        },
    }
    traffic, source = load_traffic("segscan_i8_2p%d_%s" % (args.log2n, args.variant))
    if args.density is None:
        line["roofline"]["traffic"] = traffic
        line["roofline"]["traffic_source"] = source
    else:
        line["roofline"]["traffic_source"] = "not measured for this flag density"
    if not args.no_cpu_baseline:
        import oracle
        secs, ref = oracle_baseline(x, f)
        # the output of the last timed step against the oracle's (bit-exact: integers)
        got = zt.cpu().numpy()
        assert np.array_equal(got, ref), "the timed run's output differs from the oracle's"
        line["config"]["output_checked_against_oracle"] = True
        del got, ref
        line["cpu_baseline"] = {
            "value": n / secs / 1e9,
            "unit": "Gelem/s",
            "cores": 1,
            "kind": "oracle",
            "sample": "the whole n=2^%d workload, sequential C loop (gcc -O2), best of 3 runs, "
                      "host has %d logical CPUs" % (args.log2n, os.cpu_count()),
        }
        threads = min(os.cpu_count() or 1, 256)
        secs_t = None
        for _ in range(3):
            t0 = time.perf_counter()
            oracle.host_threads_segscan(x, f, threads)
            secs_t = min(secs_t or 1e30, time.perf_counter() - t0)
        line["cpu_all_cores"] = {
            "value": n / secs_t / 1e9,
            "unit": "Gelem/s",
            "cores": threads,
            "kind": "chunked three-step scan on host threads (not the oracle; checked against it)",
            "sample": "the whole n=2^%d workload, best of 3 runs" % args.log2n,
        }
    del copies[1:]
    if args.report:
        write_report(args, events)
    print(json.dumps(line))
    return 0


# ---- the wider report (not part of the contract line) -------------------------------------------------------

def write_report(args, events: HipEvents) -> None:
    import torch
    from paper_2506_23906_amd import binding as B
    from paper_2506_23906_amd import workloads as W
    rows = []

    def emit(**kw):
        rows.append(kw)
        print("[report] " + json.dumps(kw), file=sys.stderr, flush=True)

    def copy_rate(in_bytes: int, out_bytes: int, steps=50):
        src = torch.empty(max(in_bytes, 16), dtype=torch.uint8, device="cuda").zero_()
        dst = torch.empty(max(out_bytes, 16), dtype=torch.uint8, device="cuda")
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(5):
            B.mmv_stream_copy(src, dst, in_bytes, out_bytes)
        a.record()
        for _ in range(steps):
            B.mmv_stream_copy(src, dst, in_bytes, out_bytes)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / steps
        return (in_bytes + out_bytes) / (ms * 1e-3) / 1e9, ms

    def call_ms(fn, steps=30, warmup=3):
        """Whole call (reset kernels included) timed with stream events; mean over `steps`."""
        for _ in range(warmup):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / steps

    def run(name, n, algo_bytes, step, ws, steps=args.steps):
        wall, kern = time_steps(step, steps, args.warmup, events)
        assert B.mmv_workspace_status(ws) == 0
        emit(workload=name, n=n, ms_per_step=wall, kernel_ms=kern, gelem_s=n / (wall * 1e-3) / 1e9,
             algo_bytes=algo_bytes, gb_s_kernel=algo_bytes / (kern * 1e-3) / 1e9,
             frac_of_peak_kernel=algo_bytes / (kern * 1e-3) / 1e9 / HBM_PEAK_GBS)

    # copy references: 1:4 (int8 -> int32), 1:1 (fp32 -> fp32), read only
    for label, ib, ob in [("copy 1B:4B, 256 MiB in", 1 << 28, 1 << 30), ("copy 4B:4B, 1 GiB in", 1 << 30, 1 << 30),
                          ("read only, 1 GiB", 1 << 30, 0), ("write only, 1 GiB", 0, 1 << 30)]:
        gbs, ms = copy_rate(ib, ob)
        emit(workload=label, ms=ms, gb_s=gbs, frac_of_peak=gbs / HBM_PEAK_GBS)

    # workload 1
    x, f = W.scan_sum_f32_bernoulli()
    n = len(x)
    xt, ft = torch.from_numpy(x).cuda(), torch.from_numpy(W.pack_flags(f).view(np.int32)).cuda()
    for variant in ("mfma", "shuffle"):
        zt = torch.empty(n, dtype=torch.float32, device="cuda")
        ws = B.new_workspace(B.MMV_OP_SEGSCAN, B.MMV_F32_F32, B.MMV_FLAGS_PACKED32, n)
        run("1 segscan f32 n=2^16 bernoulli(1/64) " + variant, n, n * 8 + n // 8,
            lambda: B.mmv_segscan(xt, ft, n=n, z=zt, variant=variant, ws=ws), ws)
        out = torch.empty(n, dtype=torch.float32, device="cuda")
        nseg = torch.empty(1, dtype=torch.int64, device="cuda")
        ws2 = B.new_workspace(B.MMV_OP_SEGSUM, B.MMV_F32_F32, B.MMV_FLAGS_PACKED32, n)
        run("1 segsum f32 n=2^16 bernoulli(1/64) " + variant, n, n * 4 + n // 8 + int(f.sum()) * 4,
            lambda: B.mmv_segsum(xt, ft, n=n, out=out, nseg=nseg, variant=variant, ws=ws2), ws2)

    # workload 2
    x, f = W.segsum_f16_geometric()
    n = len(x)
    xt, ft = torch.from_numpy(x).cuda(), torch.from_numpy(W.pack_flags(f).view(np.int32)).cuda()
    nsegs = int(f.sum())
    for variant in ("mfma", "shuffle"):
        out = torch.empty(nsegs + 16, dtype=torch.float32, device="cuda")
        nseg = torch.empty(1, dtype=torch.int64, device="cuda")
        ws = B.new_workspace(B.MMV_OP_SEGSUM, B.MMV_F16_F32, B.MMV_FLAGS_PACKED32, n)
        run("2 segsum f16 n=2^24 geometric(32) " + variant, n, n * 2 + n // 8 + nsegs * 4,
            lambda: B.mmv_segsum(xt, ft, n=n, out=out, nseg=nseg, variant=variant, ws=ws), ws)
    # the rows above read the same 34 MiB every call, which the 256 MiB memory-side cache may hold; the next one
    # rotates over nine copies (306 MiB) so that no call finds its inputs cached
    cold = [(xt, ft)] + [(xt.clone(), ft.clone()) for _ in range(8)]
    turn = [0]

    def cold_step():
        xk, fk = cold[turn[0] % len(cold)]
        turn[0] += 1
        B.mmv_segsum(xk, fk, n=n, out=out, nseg=nseg, ws=ws)

    run("2 segsum f16 n=2^24 geometric(32) mfma, inputs rotated over 9 copies (not cached)", n,
        n * 2 + n // 8 + nsegs * 4, cold_step, ws)
    del cold

    # workload 3, both variants, and a flag-density sweep on the same values
    x, f = W.segscan_i8_uniform_len(1 << args.log2n)
    n = len(x)
    xt, ft = torch.from_numpy(x).cuda(), torch.from_numpy(W.pack_flags(f).view(np.int32)).cuda()
    zt = torch.empty(n, dtype=torch.int32, device="cuda")
    ws = B.new_workspace(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
    for variant in ("mfma", "shuffle"):
        run("3 segscan i8 n=2^%d U{1..4096} %s" % (args.log2n, variant), n, n * 5 + n // 8,
            lambda: B.mmv_segscan(xt, ft, n=n, z=zt, variant=variant, ws=ws), ws)
    # the same call with one flag byte per element (the paper's flag format): a packing kernel runs first
    f8 = torch.from_numpy(f).cuda()
    ws8 = B.new_workspace(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, B.MMV_FLAGS_U8, n)
    ms = call_ms(lambda: B.mmv_segscan(xt, f8, n=n, z=zt, ws=ws8))
    emit(workload="3 segscan i8 n=2^%d U{1..4096}, one flag byte per element (whole call)" % args.log2n, n=n, ms=ms,
         gelem_s=n / ms / 1e6, gb_s=n * 6 / ms / 1e6, frac_of_peak=n * 6 / ms / 1e6 / HBM_PEAK_GBS)
    del f8, ws8
    # (the densities of the paper's figure on segmented scan against flag density, Sec. 5.2.2: 0.01 % to 1 %, for int8
    # and fp16 inputs; 0, 10 % and 100 % added)
    densities = (0.0, 1e-4, 1e-3, 3e-3, 5e-3, 1e-2, 0.1, 1.0)
    xh = xt.to(torch.float16)
    zf = zt.view(torch.float32)
    wsh = B.new_workspace(B.MMV_OP_SEGSCAN, B.MMV_F16_F32, B.MMV_FLAGS_PACKED32, n)
    for density in densities:
        fd = torch.from_numpy(W.pack_flags(W.uniform_density_flags(n, density, 77)).view(np.int32)).cuda()
        for variant in ("mfma", "shuffle"):
            run("density sweep i8 n=2^%d density=%g %s" % (args.log2n, density, variant), n, n * 5 + n // 8,
                lambda: B.mmv_segscan(xt, fd, n=n, z=zt, variant=variant, ws=ws), ws, steps=30)
        run("density sweep f16 n=2^%d density=%g mfma" % (args.log2n, density), n, n * 6 + n // 8,
            lambda: B.mmv_segscan(xh, fd, n=n, z=zf, ws=wsh), wsh, steps=30)
    # segmented sum on the same values at the densities of the paper's breakdown, every input type, both variants
    nseg_t = torch.empty(1, dtype=torch.int64, device="cuda")
    for density in (1e-3, 1e-2):
        fd_np = W.uniform_density_flags(n, density, 78)
        ns = int(fd_np.sum()) + (0 if fd_np[0] else 1)
        fd = torch.from_numpy(W.pack_flags(fd_np).view(np.int32)).cuda()
        for label, xin, dt, width in (("i8", xt, B.MMV_I8_I32, 1), ("f16", xh, B.MMV_F16_F32, 2), ("f32", None, B.MMV_F32_F32, 4)):
            xin = xt.to(torch.float32) if xin is None else xin
            out = torch.empty(ns + 16, dtype=torch.int32 if label == "i8" else torch.float32, device="cuda")
            wss = B.new_workspace(B.MMV_OP_SEGSUM, dt, B.MMV_FLAGS_PACKED32, n)
            for variant in ("mfma", "shuffle"):
                run("segsum %s n=2^%d density=%g %s" % (label, args.log2n, density, variant), n, n * width + n // 8 + ns * 4,
                    lambda: B.mmv_segsum(xin, fd, n=n, out=out, nseg=nseg_t, variant=variant, ws=wss), wss, steps=30)
            del xin, out, wss
    # another group on the same kernel: bytes under bit-wise exclusive or (the matrix-core variant takes the running
    # xor as the parity of integer sums, two bit planes per product)
    xu = torch.from_numpy(np.random.default_rng(2390692).integers(0, 256, size=n, dtype=np.uint8)).cuda()
    wsx = B.new_workspace(B.MMV_OP_SEGSCAN, B.MMV_U8_XOR, B.MMV_FLAGS_PACKED32, n)
    for variant in ("mfma", "shuffle"):
        run("xor segscan u8 n=2^%d U{1..4096} %s" % (args.log2n, variant), n, n * 5 + n // 8,
            lambda: B.mmv_segscan(xu, ft, n=n, z=zt, variant=variant, ws=wsx), wsx, steps=30)
    del xt, ft, zt, xh, zf, xu

    # workload 4
    nr = 1 << 20
    row, col, val, xv = W.spmv_coo_zipf(nr, nr, 1 << 25)
    nnz = len(val)
    rt, ct, vt, xvt = (torch.from_numpy(a).cuda() for a in (row, col, val, xv))
    yt = torch.empty(nr, dtype=torch.float32, device="cuda")
    ws = B.new_workspace(B.MMV_OP_SPMV_COO, B.MMV_F32_F32, B.MMV_FLAGS_PACKED32, nnz)
    for variant in ("mfma", "shuffle"):
        run("4 spmv coo 2^20 x 2^20 nnz=%d zipf(1.5) %s" % (nnz, variant), nnz, nnz * 12 + 2 * nr * 4,
            lambda: B.mmv_spmv_coo(nr, nr, rt, ct, vt, xvt, y=yt, variant=variant, ws=ws), ws)
    # the same product in two steps: the flags made once (mmv_spmv_coo_prepare), every timed call the product alone
    B.mmv_spmv_coo_prepare(nr, nr, rt, ct, ws=ws)
    ms = call_ms(lambda: B.mmv_spmv_coo_run(nr, nr, rt, ct, vt, xvt, ws, y=yt))
    emit(workload="4 spmv coo, prepared matrix (mmv_spmv_coo_run, whole call)", nnz=nnz, ms=ms, gnnz_s=nnz / ms / 1e6,
         algo_bytes=nnz * 8 + nnz // 8 + 2 * nr * 4, gb_s=(nnz * 8 + nnz // 8 + 2 * nr * 4) / ms / 1e6)
    # what the random accesses to x cost on their own (val and col streamed, x[col] gathered, nothing else)
    part = torch.empty(B.GATHER_REFERENCE_PARTIALS, dtype=torch.float32, device="cuda")
    ms = call_ms(lambda: B.mmv_gather_reference(vt, ct, xvt, part))
    emit(workload="4 gather reference val*x[col] nnz=%d" % nnz, nnz=nnz, ms=ms, gnnz_s=nnz / ms / 1e6,
         algo_bytes=nnz * 8, gb_s=nnz * 8 / ms / 1e6)
    del rt, ct, vt, xvt, part

    # workload 5
    x, f = W.stress_f32_three_regimes(1 << 30)
    n = len(x)
    xt, ft = torch.from_numpy(x).cuda(), torch.from_numpy(W.pack_flags(f).view(np.int32)).cuda()
    zt = torch.empty(n, dtype=torch.float32, device="cuda")
    ws = B.new_workspace(B.MMV_OP_SEGSCAN, B.MMV_F32_F32, B.MMV_FLAGS_PACKED32, n)
    for variant in ("mfma", "shuffle"):
        run("5 stress segscan f32 n=2^30 " + variant, n, n * 8 + n // 8,
            lambda: B.mmv_segscan(xt, ft, n=n, z=zt, variant=variant, ws=ws), ws, steps=20)

    del xt, ft, zt
    torch.cuda.empty_cache()

    # unsegmented scan (Algorithm Scan) next to the segmented one, n = 2^28
    n = 1 << args.log2n
    x, _ = W.segscan_i8_uniform_len(n)
    xt = torch.from_numpy(x).cuda()
    zt = torch.empty(n, dtype=torch.int32, device="cuda")
    ws = B.new_workspace(B.MMV_OP_SCAN, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
    for variant in ("mfma", "shuffle"):
        run("scan (unsegmented) i8 n=2^%d %s" % (args.log2n, variant), n, n * 5,
            lambda: B.mmv_scan(xt, n=n, z=zt, variant=variant, ws=ws), ws, steps=30)
    xh = torch.from_numpy(np.random.default_rng(3).standard_normal(n, dtype=np.float32).astype(np.float16)).cuda()
    zf = zt.view(torch.float32)
    wsh = B.new_workspace(B.MMV_OP_SCAN, B.MMV_F16_F32, B.MMV_FLAGS_PACKED32, n)
    for variant in ("mfma", "shuffle"):
        run("scan (unsegmented) f16 n=2^%d %s" % (args.log2n, variant), n, n * 6,
            lambda: B.mmv_scan(xh, n=n, z=zf, variant=variant, ws=wsh), wsh, steps=30)
    del xh
    xf = torch.from_numpy(np.random.default_rng(4).standard_normal(n, dtype=np.float32)).cuda()
    ws32 = B.new_workspace(B.MMV_OP_SCAN, B.MMV_F32_F32, B.MMV_FLAGS_PACKED32, n)
    for variant in ("mfma", "shuffle"):
        run("scan (unsegmented) f32 n=2^%d %s" % (args.log2n, variant), n, n * 8,
            lambda: B.mmv_scan(xf, n=n, z=zf, variant=variant, ws=ws32), ws32, steps=30)
    del xf, zf

    # the primitives of Algorithms SCD / SSCR one by one, the un-fused compositions and the fused
    # calls, on uniformly random flags at the densities the paper's breakdown uses
    for density in (1e-3, 1e-2):
        f = W.uniform_density_flags(n, density, 78)
        fm = np.concatenate([f[1:], np.ones(1, dtype=np.uint8)])
        nseg = int(f.sum())
        ft = torch.from_numpy(W.pack_flags(f).view(np.int32)).cuda()
        fmt = torch.from_numpy(W.pack_flags(fm).view(np.int32)).cuda()
        f8 = torch.from_numpy(f.view(np.int8)).cuda()
        xhat = torch.empty(n, dtype=torch.int32, device="cuda")
        fhat = torch.empty(n, dtype=torch.int32, device="cuda")
        w = torch.empty(nseg + 16, dtype=torch.int32, device="cuda")
        cnt = torch.empty(1, dtype=torch.int64, device="cuda")
        out = torch.empty(nseg + 16, dtype=torch.int32, device="cuda")
        wsc = B.new_workspace(B.MMV_OP_COMPRESS, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
        tag = "n=2^%d i8 density=%g" % (args.log2n, density)

        def prim(name, fn, algo_bytes):
            ms = call_ms(fn)
            emit(workload="primitive %s %s" % (name, tag), n=n, ms=ms, gelem_s=n / ms / 1e6, algo_bytes=algo_bytes,
                 gb_s=algo_bytes / ms / 1e6, frac_of_peak=algo_bytes / ms / 1e6 / HBM_PEAK_GBS)
            return ms

        t_scan = prim("SCAN(x) int8->int32", lambda: B.mmv_scan(xt, n=n, z=xhat, ws=ws), n * 5)
        t_scanf = prim("SCAN(f) int8->int32", lambda: B.mmv_scan(f8, n=n, z=fhat, ws=ws), n * 5)
        t_comp = prim("COMPRESS(xhat, f-)", lambda: B.mmv_compress(xhat, fmt, n, out=w, count=cnt, ws=wsc),
                      n // 8 + nseg * 8)
        t_diff = prim("DIFF(w)", lambda: B.mmv_diff(w, n=nseg, z=out), nseg * 8)
        # SCAN(f) of flags that hold a 1 at position 0 is the count REVERT needs
        t_rev = prim("REVERT", lambda: B.mmv_revert(xhat, fhat, w, n=n, nw=nseg, z=zt), n * 12)
        wsd = B.new_workspace(B.MMV_OP_SEGSUM_SCD, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
        nsg = torch.empty(1, dtype=torch.int64, device="cuda")
        t_scd = prim("SCD un-fused (segsum)", lambda: B.mmv_segsum_scd(xt, ft, n=n, out=out, nseg=nsg, ws=wsd),
                     n + n // 8 + nseg * 4)
        del wsd
        wss = B.new_workspace(B.MMV_OP_SEGSUM, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
        t_sum = prim("fused mmv_segsum", lambda: B.mmv_segsum(xt, ft, n=n, out=out, nseg=nsg, ws=wss),
                     n + n // 8 + nseg * 4)
        wsr = B.new_workspace(B.MMV_OP_SEGSCAN_SSCR, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
        t_sscr = prim("SSCR un-fused (segscan)", lambda: B.mmv_segscan_sscr(xt, ft, n=n, z=zt, ws=wsr), n * 5 + n // 8)
        del wsr
        wsg = B.new_workspace(B.MMV_OP_SEGSCAN, B.MMV_I8_I32, B.MMV_FLAGS_PACKED32, n)
        t_seg = prim("fused mmv_segscan", lambda: B.mmv_segscan(xt, ft, n=n, z=zt, ws=wsg), n * 5 + n // 8)
        emit(workload="fusion summary " + tag, scd_over_fused=t_scd / t_sum, sscr_over_fused=t_sscr / t_seg,
             compress_share_of_scd=t_comp / (t_scan + t_comp + t_diff),
             compress_share_of_sscr=t_comp / (t_scan + t_scanf + t_comp + t_rev),
             revert_share_of_sscr=t_rev / (t_scan + t_scanf + t_comp + t_rev))
        del ft, fmt, f8, xhat, fhat, w, out
    del xt, zt
    torch.cuda.empty_cache()

    # CSR SpMV: workload 4 through its row pointers, and the blocked sparse-attention matrices
    rowptr = W.csr_rowptr(row, nr)
    rpt, ct, vt, xvt = (torch.from_numpy(a).cuda() for a in (rowptr, col, val, xv))
    wsv = torch.empty(B.mmv_spmv_csr_workspace_bytes(nr, nnz), dtype=torch.uint8, device="cuda")
    ms = call_ms(lambda: B.mmv_spmv_csr(nr, nr, rpt, ct, vt, xvt, y=yt, ws=wsv))
    emit(workload="4 spmv csr 2^20 x 2^20 nnz=%d zipf(1.5)" % nnz, nnz=nnz, ms=ms, gnnz_s=nnz / ms / 1e6,
         algo_bytes=nnz * 8 + 3 * nr * 4, gb_s=(nnz * 8 + 3 * nr * 4) / ms / 1e6)
    B.mmv_spmv_csr_prepare(nr, nr, rpt, ct, ws=wsv)
    ms = call_ms(lambda: B.mmv_spmv_csr_run(nr, nr, rpt, ct, vt, xvt, wsv, y=yt))
    emit(workload="4 spmv csr, prepared matrix (mmv_spmv_csr_run, whole call)", nnz=nnz, ms=ms, gnnz_s=nnz / ms / 1e6,
         algo_bytes=nnz * 8 + nnz // 8 + 2 * nr * 4, gb_s=(nnz * 8 + nnz // 8 + 2 * nr * 4) / ms / 1e6)
    del rpt, ct, vt, xvt, wsv
    na = 1 << 16
    for block in (2, 4, 16, 64):
        for n_random in (2, 4, 8):
            rp, c, v, xa = W.blocked_sparse_attention(na, block=block, n_random=n_random)
            nz = len(v)
            rpt, ct, vt, xat = (torch.from_numpy(a).cuda() for a in (rp, c, v, xa))
            ya = torch.empty(na, dtype=torch.float32, device="cuda")
            wsv = torch.empty(B.mmv_spmv_csr_workspace_bytes(na, nz), dtype=torch.uint8, device="cuda")
            ms = call_ms(lambda: B.mmv_spmv_csr(na, na, rpt, ct, vt, xat, y=ya, ws=wsv))
            emit(workload="spmv csr sparse attention 65536^2 b-%d_r-%d" % (block, n_random), nnz=nz, ms=ms,
                 gnnz_s=nz / ms / 1e6, algo_bytes=nz * 8 + 3 * na * 4, gb_s=(nz * 8 + 3 * na * 4) / ms / 1e6)
            if n_random == 8:
                B.mmv_spmv_csr_prepare(na, na, rpt, ct, ws=wsv)
                ms = call_ms(lambda: B.mmv_spmv_csr_run(na, na, rpt, ct, vt, xat, wsv, y=ya))
                emit(workload="spmv csr sparse attention 65536^2 b-%d_r-%d, prepared matrix" % (block, n_random), nnz=nz, ms=ms,
                     gnnz_s=nz / ms / 1e6, algo_bytes=nz * 8 + nz // 8 + 2 * na * 4, gb_s=(nz * 8 + nz // 8 + 2 * na * 4) / ms / 1e6)
                part = torch.empty(B.GATHER_REFERENCE_PARTIALS, dtype=torch.float32, device="cuda")
                ms = call_ms(lambda: B.mmv_gather_reference(vt, ct, xat, part))
                emit(workload="gather reference sparse attention 65536^2 b-%d_r-%d" % (block, n_random), nnz=nz, ms=ms,
                     gnnz_s=nz / ms / 1e6, algo_bytes=nz * 8, gb_s=nz * 8 / ms / 1e6)

    with open(args.report, "w") as fh:
        for r in rows:
            fh.write(json.dumps(r) + "\n")


if __name__ == "__main__":
    sys.exit(main())
