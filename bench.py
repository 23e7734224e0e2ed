#!/usr/bin/env python3
"""Benchmark of the device-wide scan on one MI355X.

A step is one pass of the whole hot path (one ks_scan call: load, register scan, wave scan, LDS
exchange, look-back, store) over one batch of synthetic input that is already resident in HBM.
Default workload: the headline configuration, inclusive float32 sum scan of n = 2^28
values uniform in [0, 1) from seed 1.  Prints ONE JSON line on stdout; everything else goes to
stderr.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--n N] [--stride S]
                    [--mapreduce [--map MAP]] [--no-cpu]

With --stride S > 1 (scalar workloads) the same elements sit S elements apart in both buffers and
ks_scan_strided runs; GB/s still counts the elements alone (2 * n * element size).
With --mapreduce the step is one ks_mapreduce call (the workload's operator, the map of --map) on the same
input, and GB/s counts n * element size: every element read once, one element written.  The workload
u8_codes (uint8 codes; maps unit_float8, widen64 or identity) exists for --mapreduce only.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak


TRAFFIC_SUMMARY = os.path.join("profiles", "scan_lookback_f32_sum_2p28_hbm_traffic.md")


def measured_traffic(workload: str, n: int):
    """HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary, for the
    headline configuration only (None for anything else, or when the summary is absent).  Counters
    cannot be read from inside a run: the figure is the one the profiler measured for this kernel."""
    if workload != "f32_sum" or n != 1 << 28:
        return None
    try:
        for line in open(os.path.join(ROOT, TRAFFIC_SUMMARY)):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


# the oracle's names for the workloads' (operator, element type): only the oracle leg uses them
ORACLE_KIND = {"int32_sum": ("sum", "i32"), "f32_sum": ("sum", "f32"), "u64_exsum": ("sum", "u64"),
               "affine": ("affine", "f32"), "argmax": ("argmax", None), "f64_sum": ("sum", "f64"), "u8_codes": ("sum", "u64"),
               "bf16_sum": ("sum", "f32"), "f16_sum": ("sum", "f32")}
HALF_KINDS = {"bf16_sum": ("bf16", 7, -126), "f16_sum": ("f16", 10, -14)}    # oracle's name, mantissa bits, lowest exponent
FLOAT_WORKLOADS = {"f32_sum", "affine", "f64_sum"}
PREHEAT_S = 0.1


def worst_ratio_or_raise(workload: str, got, ref, what: str) -> float:
    """The parity bar of the GPU tests, applied to one chunk: bit-exact for integer and struct
    workloads, |gpu - ref| <= max(1e-4 |ref|, 1e-3) against the oracle's float64 result for float ones."""
    if workload in FLOAT_WORKLOADS:
        err = np.abs(got.astype(np.float64).reshape(ref.shape) - ref)
        ratio = float(np.max(err / np.maximum(1e-4 * np.abs(ref), 1e-3))) if err.size else 0.0
        if not ratio <= 1.0:
            raise AssertionError(f"{what}: float mismatch, worst ratio {ratio:.3g}")
        return ratio
    if got.tobytes() != ref.tobytes():
        raise AssertionError(f"{what}: integer results differ from the oracle")
    return 0.0


def half_ratio_or_raise(workload: str, got_bits, ref, what: str) -> float:
    """16-bit float outputs of a sum scan against the oracle's float64 values: within half a unit in the
    last place of the 16-bit type plus the float bar of the float32 accumulation (the GPU tests' bar)."""
    import oracle
    kind, mantissa, low = HALF_KINDS[workload]
    got = oracle.apply_map("widen_f32", got_bits, kind).astype(np.float64)
    half_ulp = 0.5 * 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** low))) - mantissa)
    ratio = float(np.max(np.abs(got - ref) / (half_ulp + np.maximum(1e-4 * np.abs(ref), 1e-3)))) if len(ref) else 0.0
    if not ratio <= 1.0:
        raise AssertionError(f"{what}: 16-bit outputs off, worst ratio {ratio:.3g}")
    return ratio


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="f32_sum")
    ap.add_argument("--n", type=int, default=0)
    ap.add_argument("--algo", default="auto", choices=["auto", "lookback", "reduce_then_scan"])
    ap.add_argument("--stride", type=int, default=1, help="element stride of both views (ks_scan_strided)")
    ap.add_argument("--mapreduce", action="store_true", help="time ks_mapreduce (reads n elements) instead of the scan")
    ap.add_argument("--map", default="identity", help="with --mapreduce: the map f of mapreduce(f, op, src), e.g. "
                    "unit_float8 or widen64 for --workload u8_codes")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle leg (cpu_baseline = null)")
    ap.add_argument("--preheat-s", type=float, default=PREHEAT_S, help="seconds of plain copies before the warm-up "
                    "steps (the clocks drop while the host prepares the inputs); untimed, reported as preheat_s")
    ap.add_argument("--opt", action="append", default=[], help="library option name=value (tuning runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build measures one GPU only (the scan's cross-GPU sharding is a design note, "
            "not code); run with --gpus 1")
        return 2

    import torch
    import ks_inputs
    import paper_2603_18695_amd as ks
    from ks_marshal import to_device, to_host

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the scan has no CPU fallback")
        return 2
    torch.cuda.set_device(0)
    for kv in args.opt:
        k, v = kv.split("=")
        ks.ks_set_option(k, int(v))

    w = ks_inputs.WORKLOADS[args.workload]
    n = args.n or (w.n if args.workload != "argmax" else 1 << 26)
    eb = w.elem_bytes
    # every element read once and written once; a reduction only reads
    algorithmic_bytes = n * eb if args.mapreduce else 2 * n * eb
    if args.mapreduce and (args.stride > 1 or args.algo != "auto"):
        log("bench.py: --mapreduce goes with --stride 1 and --algo auto")
        return 2
    if not args.mapreduce and (args.map != "identity" or w.dtype == "u8"):
        log("bench.py: --map and the byte workload go with --mapreduce (the scans take neither)")
        return 2
    if args.mapreduce and w.dtype in ("bf16", "f16") and args.map == "identity":
        args.map = "widen_f32"      # the one map under which 16-bit floats are reduced
    if args.mapreduce and not ks.ks_mapreduce_result_bytes(dtype=w.dtype, op=w.op, map=args.map):
        log(f"bench.py: ks_mapreduce does not take ({w.dtype}, {args.map}, {w.op})")
        return 2

    # ---- inputs: generated on the host from the seeded recipe, then resident in HBM
    t0 = time.time()
    host_chunks = list(ks_inputs.chunks(args.workload, n))
    d_in = torch.cat([to_device(c) for c in host_chunks])
    d_out = torch.empty_like(d_in)
    temp = torch.empty(ks.ks_scan_temp_bytes(dtype=w.dtype, op=w.op, n=n, algo=args.algo), dtype=torch.uint8,
                       device="cuda")
    log(f"inputs: workload={args.workload} n={n} ({n * eb / 2**20:.0f} MiB each way) generated in {time.time() - t0:.1f}s")

    if args.stride > 1:
        if d_in.dim() != 1 or args.algo != "auto":
            log("bench.py: --stride applies to the scalar workloads with --algo auto")
            return 2
        s_in = torch.zeros(n * args.stride, dtype=d_in.dtype, device="cuda")
        s_in[::args.stride] = d_in
        s_out = torch.zeros_like(s_in)

    d_one = torch.empty_like(d_in[:1])
    if args.mapreduce:    # one element of the result type, which a map may have changed
        d_one = torch.empty(ks.ks_mapreduce_result_bytes(dtype=w.dtype, op=w.op, map=args.map), dtype=torch.uint8,
                            device="cuda")

    def step():
        if args.mapreduce:
            ks.ks_mapreduce(d_in, d_one, dtype=w.dtype, op=w.op, map=args.map)
        elif args.stride > 1:
            ks.ks_scan_strided(s_in, s_out, dtype=w.dtype, op=w.op, n=n, in_stride=args.stride,
                               out_stride=args.stride, inclusive=w.inclusive)
        elif args.algo == "auto":
            ks.ks_scan(d_in, d_out, dtype=w.dtype, op=w.op, inclusive=w.inclusive)
        else:
            ks.ks_scan_with_temp(d_in, d_out, temp, dtype=w.dtype, op=w.op, inclusive=w.inclusive, algo=args.algo)

    # The GPU's clocks drop while the host generates and copies the inputs (a scan right after reads
    # up to 7 % low for some tens of milliseconds): keep the memory system busy for 0.1 s with the
    # plain copy kernel first.  Not part of the W warm-up steps, which follow, nor of the timed region.
    t_busy = time.perf_counter()
    while time.perf_counter() - t_busy < args.preheat_s:
        for _ in range(20):
            ks.ks_copy(d_in, d_out)
        torch.cuda.synchronize()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ks.ks_scan_check()

    # ---- timed region: exactly K steps, sync on both sides; HIP events on the launch stream
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    ks.ks_scan_check()
    wall_ms = (t_end - t_start) * 1e3 / args.steps
    event_ms = ev0.elapsed_time(ev1) / args.steps
    gbs_wall = algorithmic_bytes / (wall_ms * 1e-3) / 1e9
    gbs_event = algorithmic_bytes / (event_ms * 1e-3) / 1e9
    log(f"scan: {wall_ms:.4f} ms/step wall, {event_ms:.4f} ms/step by HIP events -> {gbs_event:.1f} GB/s "
        f"({100 * gbs_event / HBM_PEAK_GBS:.1f}% of {HBM_PEAK_GBS:.0f} GB/s)")

    # ---- the paper's protocol (Sec. VII: one launch per event pair, mean +- std; launch overhead
    #      included), outside the timed region
    singles = []
    for _ in range(0 if args.no_cpu else 50):   # not in the short runs that the profiles are taken from
        s0 = torch.cuda.Event(enable_timing=True)
        s1 = torch.cuda.Event(enable_timing=True)
        s0.record()
        step()
        s1.record()
        torch.cuda.synchronize()
        singles.append(s0.elapsed_time(s1) * 1e3)
    ks.ks_scan_check()
    launch_stats = None
    if singles:
        launch_stats = {"launches": len(singles), "mean_us": float(np.mean(singles)), "std_us": float(np.std(singles)),
                        "min_us": float(np.min(singles)), "max_us": float(np.max(singles))}
        log(f"single launches: {launch_stats['mean_us']:.1f} +- {launch_stats['std_us']:.1f} us (min {launch_stats['min_us']:.1f})")

    # ---- copy kernel on the same bytes: the practical ceiling (context, not the metric)
    for _ in range(5):
        ks.ks_copy(d_in, d_out)
    torch.cuda.synchronize()
    c0 = torch.cuda.Event(enable_timing=True)
    c1 = torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(50):
        ks.ks_copy(d_in, d_out)
    c1.record()
    torch.cuda.synchronize()
    copy_ms = c0.elapsed_time(c1) / 50
    copy_gbs = 2 * n * eb / (copy_ms * 1e-3) / 1e9      # the copy reads and writes n elements
    log(f"copy ceiling: {copy_ms:.4f} ms -> {copy_gbs:.1f} GB/s")

    # ---- oracle leg: the sequential CPU scan on this host, one core, and a parity check of the
    #      result the timed configuration produced
    cpu = None
    parity = None
    if not args.no_cpu:
        import oracle
        step()
        torch.cuda.synchronize()
        if args.stride > 1:
            d_out = s_out[::args.stride].contiguous()
        oop, odt = ORACLE_KIND[args.workload]
        if args.mapreduce:    # the fold runs over the mapped elements, in the type the map gives them
            odt = {"unit_float8": "f32", "widen64": "u64", "widen_f32": "f32"}.get(args.map, "u64" if w.dtype == "u8" else odt)
            if args.map == "square" and odt == "f32":
                odt = "f64"
        budget_elems = n if w.dtype == "u8" else min(n, 1 << 28)
        stream = oracle.ScanStream(oop, odt, True if args.mapreduce else w.inclusive)
        cpu_s, done, at, worst = 0.0, 0, 0, 0.0
        for c in host_chunks:
            if done >= budget_elems:
                break
            t = time.perf_counter()
            bits = c
            if args.workload in HALF_KINDS:      # the 16-bit floats are promoted (exactly) before the fold
                c = oracle.apply_map("widen_f32", c, HALF_KINDS[args.workload][0])
            elif args.mapreduce and (args.map != "identity" or w.dtype == "u8"):
                c = oracle.apply_map("widen64" if (w.dtype, args.map) == ("u8", "identity") else args.map, c)
            ref = stream.feed(c)
            cpu_s += time.perf_counter() - t
            if not args.mapreduce and args.workload in HALF_KINDS:
                got = to_host(d_out[at:at + len(c)], bits.dtype)
                worst = max(worst, half_ratio_or_raise(args.workload, got, ref, f"bench parity at {at}"))
            elif not args.mapreduce:
                got = to_host(d_out[at:at + len(c)], c.dtype)
                worst = max(worst, worst_ratio_or_raise(args.workload, got, ref, f"bench parity at {at}"))
            at += len(c)
            done += len(c)
        if args.mapreduce and done == n:     # the fold's last running value is the reduction
            last = ref[-1:]
            if (w.dtype, args.map) == ("u8", "identity"):
                last = (last & np.uint64(0xFF)).astype(np.uint8)      # the element type's own addition: modulo 2^8
            if w.dtype == "u8":
                got = d_one.cpu().numpy().view(np.float32 if args.map == "unit_float8" else last.dtype)
                kind = "f32_sum" if args.map == "unit_float8" else "int32_sum"    # float bar, or bit for bit
            elif args.workload in HALF_KINDS:
                got, kind = d_one.cpu().numpy().view(np.float32), "f32_sum"
            else:
                got = to_host(d_one.view(d_in.dtype).reshape((1,) + tuple(d_in.shape[1:])), host_chunks[0].dtype)
                kind = args.workload
            worst = worst_ratio_or_raise(kind, got, last, "bench parity, mapreduce")
        parity = {"checked_elements": done, "worst_float_ratio": worst}
        cpu_gbs = (1 if args.mapreduce else 2) * done * eb / cpu_s / 1e9
        cpu = {"value": cpu_gbs, "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"first {done} elements of the same workload, sequential C left fold (fp64 accumulator "
                         f"for float inputs), {cpu_s:.2f} s on {os.cpu_count()} visible host cpus, 1 thread used",
               "elements_per_s": done / cpu_s}
        log(f"oracle: {done} elements in {cpu_s:.2f}s -> {cpu_gbs:.2f} GB/s on 1 core; parity ok (worst ratio {worst:.3f})")

    # ---- the other benchmark configurations, for context in the same run (HIP events, 50 launches each;
    #      their parity is the GPU tests' business).  Only with the default workload and the oracle leg on.
    others = None
    if (not args.no_cpu and args.workload == "f32_sum" and not args.n and args.algo == "auto" and not args.opt
            and args.stride == 1 and not args.mapreduce):
        del d_in, d_out, temp
        others = {}

        def time_config(name, on):
            ow = ks_inputs.WORKLOADS[name]
            first = next(iter(ks_inputs.chunks(name, min(on, ks_inputs.CHUNK))))
            o_in = torch.empty((on,) + tuple(to_device(first[:1]).shape[1:]), dtype=to_device(first[:1]).dtype, device="cuda")
            at = 0
            for c in ks_inputs.chunks(name, on):        # chunk by chunk: 2^30 structs never exist on the host at once
                o_in[at:at + len(c)] = to_device(c)
                at += len(c)
            o_out = torch.empty_like(o_in)
            launches = 50 if on <= 1 << 28 else 10
            for _ in range(30 if on <= 1 << 28 else 5):   # the clocks drop while the inputs are generated and copied
                ks.ks_scan(o_in, o_out, dtype=ow.dtype, op=ow.op, inclusive=ow.inclusive)
            torch.cuda.synchronize()
            o0, o1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            o0.record()
            for _ in range(launches):
                ks.ks_scan(o_in, o_out, dtype=ow.dtype, op=ow.op, inclusive=ow.inclusive)
            o1.record()
            torch.cuda.synchronize()
            ks.ks_scan_check()
            oms = o0.elapsed_time(o1) / launches
            ogbs = 2 * on * ow.elem_bytes / (oms * 1e-3) / 1e9
            log(f"{name}: n={on} {oms * 1e3:.1f} us/step -> {ogbs:.1f} GB/s")
            return {"n": on, "ms_per_step": oms, "gbs": ogbs, "pct_of_hbm_peak": 100 * ogbs / HBM_PEAK_GBS,
                    "launches": launches}

        for name in ("int32_sum", "u64_exsum", "affine"):
            others[name] = time_config(name, ks_inputs.WORKLOADS[name].n)
        others["argmax"] = time_config("argmax", 1 << 26)
        others["argmax_sweep"] = [time_config("argmax", on) for on in ks_inputs.ARGMAX_SWEEP if on != 1 << 26]

    result = {
        "metric": f"mapreduce GB/s (read), workload {args.workload}{'' if args.map == 'identity' else ' map ' + args.map} n={n}, "
                  "1 MI355X" if args.mapreduce
                  else "scan GB/s (read+write), float32 inclusive sum n=2^28, 1 MI355X"
                  if args.workload == "f32_sum" and n == 1 << 28 and args.stride == 1
                  else f"scan GB/s (read+write), workload {args.workload} n={n}"
                       f"{'' if args.stride == 1 else f' element stride {args.stride}'}, 1 MI355X",
        "value": gbs_wall,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "preheat_s": args.preheat_s,   # plain copies before the warm-up steps, to bring the clocks up; not timed
        "ms_per_step": wall_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"f32_sum": "f32", "int32_sum": "i32", "u64_exsum": "u64", "affine": "f64", "argmax": "i32/i64",
                  "f64_sum": "f64", "bf16_sum": "f32", "f16_sum": "f32", "u8_codes": {"unit_float8": "f32", "widen64": "u64"}.get(args.map, "u8")}[args.workload],
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {'inclusive' if w.inclusive else 'exclusive'} {w.op} scan, {w.dtype}, "
                               f"n={n}, seed {w.seed}", "algo": args.algo, "elem_bytes": eb, "stride": args.stride,
                   "options": {k: ks.ks_get_option(k) for k in ["waves", "rows", "prefetch", "form", "tickets", "wgs_per_cu"]}},
        "elements_per_s": n / (wall_ms * 1e-3),
        "pct_of_hbm_peak": 100 * gbs_wall / HBM_PEAK_GBS,
        "copy_ceiling_gbs": copy_gbs,
        "single_launch_us": launch_stats,
        "roofline": {"bound": "hbm", "achieved": gbs_event, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs_event / HBM_PEAK_GBS,
                     "traffic": measured_traffic(args.workload, n)
                                if args.algo == "auto" and not args.opt and args.stride == 1 and not args.mapreduce else None,
                     "traffic_source": f"rocprofv3 FETCH_SIZE / WRITE_SIZE of this kernel and size, read from {TRAFFIC_SUMMARY} "
                                       "(not measured in this run)",
                     "kernel_ms": event_ms, "algorithmic_bytes": algorithmic_bytes},
        "cpu_baseline": cpu,
        "parity": parity,
        "other_configs": others,
    }
    if args.mapreduce and args.map == "unit_float8":
        # five vector instructions per byte read: this reduction is bound by arithmetic before memory.
        # Peak: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second (no packed
        # float32); instructions per byte: SQ_INSTS_VALU x 64 lanes / n of this kernel, from the committed
        # rocprofv3 summary (counters cannot be read from inside a run).
        valu_per_byte, alu_peak = 5.27, 256 * 4 * 16 * 2.4e9 / 1e12
        achieved = valu_per_byte * n / (event_ms * 1e-3) / 1e12
        result["roofline"] = {"bound": "alu", "achieved": achieved, "peak": alu_peak, "unit": "T lane-instructions/s",
                              "frac": achieved / alu_peak, "traffic": None, "kernel_ms": event_ms,
                              "instructions_per_byte": valu_per_byte,
                              "instructions_source": "profiles/mapreduce_paper_sizes_f32_u8_kernel_trace.md",
                              "hbm_frac": gbs_event / HBM_PEAK_GBS}
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
