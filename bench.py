#!/usr/bin/env python3
"""Benchmark of the direct-convolution hot path on one MI355X.

A step is one launch of the single-channel kernel on the large single-channel
configuration (one 4096x4096 image, 64 filters of 5x5) with all buffers
resident in HBM.  The same JSON line also carries one entry per remaining
configuration (the small single-channel case, the filter-size sweep and the
three general-case shapes), each timed the same way, the roofline figures of
the dominant kernel, and the CPU oracle timed on a bounded sample.

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import subprocess
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP32_PEAK_TFLOPS = 157.3       # MI355X fp32 (matrix / packed vector), published
MFMA16_PEAK_TFLOPS = 2500.0    # MI355X dense fp16 / bf16 matrix cores, published
MFMA8_PEAK_TOPS = 5000.0       # MI355X dense int8 matrix cores, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-configs", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy a few times, so that a "
                         "counter run can scale FETCH_SIZE / WRITE_SIZE by a transfer of known size")
    ap.add_argument("--paper-sweep", action="store_true",
                    help="also time the other corners the paper sweeps (1x1 filters, one filter, "
                         "5x5 and 7x7 general layers, 32x32 images): entries under 'paper_sweep'")
    ap.add_argument("--no-measured-peaks", action="store_true",
                    help="do not run the hardware-rate microbenchmark whose fill and matrix-core rates "
                         "are quoted as measured achievable peaks beside the published ones")
    ap.add_argument("--only", default=None,
                    help="time just this configuration (S1, S2, S2_F3.., G1, G2, G3) as the step")
    return ap.parse_args()


def measured_peaks():
    """Rates this very box sustains, from the standalone microbenchmark built with the library
    (run as a child process before this process touches the GPU): HBM fill and read with 16 B
    per lane over 4 GiB, and the bare fp32 matrix-core loop fed from LDS.  None if it cannot run."""
    exe = ROOT / "paper_1705_10591_amd" / "hw_bench"
    if not exe.exists():
        return None
    try:
        r = subprocess.run([str(exe), "--quick"], capture_output=True, text=True, timeout=120)
    except (OSError, subprocess.TimeoutExpired):
        return None
    if r.returncode != 0:
        return None
    val = {m.group(1).strip(): float(m.group(2))
           for m in re.finditer(r"^([^#\n][^:]*):\s+[\d.]+ ms\s+([\d.]+) (?:GB/s|TFLOP/s|TOP/s)", r.stdout, re.M)}
    try:
        return {"hbm_fill_gbs": val["fill, 16 B per lane"], "hbm_read_gbs": val["read, 16 B per lane"],
                "fp32_mfma_tflops": val["no other vector instructions"],
                "bf16_mfma_tflops": val["bf16, operands from LDS every step"],
                "int8_mfma_tops": val["int8, operands from LDS every step"],
                "source": "paper_1705_10591_amd/hw_bench --quick, same box, before the timed runs"}
    except KeyError:
        return None


def add_measured(entry, peaks):
    """Fractions of the measured achievable rates beside the published-peak ones."""
    if peaks:
        entry["frac_hbm_fill_measured"] = round(entry["algorithmic_gbs"] / peaks["hbm_fill_gbs"], 4)
        entry["frac_fp32_mfma_measured"] = round(entry["gflops"] / 1e3 / peaks["fp32_mfma_tflops"], 4)
    return entry


def time_launches(fn, steps, warmup, warm_ms=0.0):
    """Average milliseconds per launch over `steps` launches, by events on the launch stream.

    `warmup` untimed launches come first; with `warm_ms` > 0 untimed launches continue until
    that much time has passed, so that short kernels are also timed at the clocks the chip
    settles at under load and not during its ramp from idle."""
    import torch
    t_start = time.perf_counter()
    done = 0
    while done < warmup or (time.perf_counter() - t_start) * 1e3 < warm_ms:
        fn()
        done += 1
        if done % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def graph_replay_ms(fn, launches=20, replays=20):
    """Per-launch time of `fn` when `launches` calls are captured into one HIP graph and the graph
    is replayed: what a launch-bound caller gets (the calls only enqueue kernels, so they can be
    captured once they have run once on the capture stream)."""
    import torch
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        fn()
    s.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        for _ in range(launches):
            fn()
    for _ in range(3):
        g.replay()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (replays * launches)


def make_runner(w):
    import torch
    import workloads as wl
    import paper_1705_10591_amd as dconv
    x, f = wl.make_inputs(w)
    xd, fd = torch.from_numpy(x).cuda(), torch.from_numpy(f).cuda()
    out = torch.empty(w.out_shape(), dtype=torch.float32, device="cuda")
    if w.kind == "single":
        return (lambda: dconv.dconv_single_channel(xd, fd, out=out)), (x, f)
    return (lambda: dconv.dconv_general(xd, fd, out=out)), (x, f)


def make_half_runner(w, kind, blocked=False):
    """The general-case shape `w` with short inputs (kind: "f16", "bf16" or "i8"), channels innermost."""
    import torch
    import workloads as wl
    from paper_1705_10591_amd import dconv_general_half, dconv_general_i8
    if kind == "i8":
        g = torch.Generator(device="cuda").manual_seed(w.seed)
        xi = torch.randint(-128, 128, (w.N, w.H, w.W, w.C), generator=g, device="cuda", dtype=torch.int8)
        fi = torch.randint(-128, 128, (w.K, w.F, w.F, w.C), generator=g, device="cuda", dtype=torch.int8)
        outi = torch.empty(w.out_shape(), dtype=torch.int32, device="cuda")
        return lambda: dconv_general_i8(xi, fi, out=outi)
    tt = torch.float16 if kind == "f16" else torch.bfloat16
    x, f = wl.make_inputs(w)
    if blocked:     # [N][C/16][H][W][16], [K][C/16][F][F][16]
        xb = torch.from_numpy(x.reshape(w.N, w.C // 16, 16, w.H, w.W)).cuda().permute(0, 1, 3, 4, 2).contiguous().to(tt)
        fb = torch.from_numpy(f.reshape(w.K, w.C // 16, 16, w.F, w.F)).cuda().permute(0, 1, 3, 4, 2).contiguous().to(tt)
        outb = torch.empty(w.out_shape(), dtype=torch.float32, device="cuda")
        return lambda: dconv_general_half(xb, fb, out=outb, blocked=True)
    xh = torch.from_numpy(x.reshape(w.N, w.C, w.H, w.W)).cuda().permute(0, 2, 3, 1).contiguous().to(tt)
    fh = torch.from_numpy(f.reshape(w.K, w.C, w.F, w.F)).cuda().permute(0, 2, 3, 1).contiguous().to(tt)
    out = torch.empty(w.out_shape(), dtype=torch.float32, device="cuda")
    return lambda: dconv_general_half(xh, fh, out=out)


def half_entry(w, kind, ms):
    gflops = w.flops / (ms * 1e-3) / 1e9
    peak = MFMA8_PEAK_TOPS if kind == "i8" else MFMA16_PEAK_TFLOPS
    return {"name": f"{w.name}_{kind}", "kernel": f"dconv_general_{kind}",
            "shape": {"N": w.N, "C": w.C, "H": w.H, "W": w.W, "K": w.K, "F": w.F},
            "layout": "in[N][H][W][C], filt[K][F][F][C], out[N][K][Ho][Wo] " + ("int32" if kind == "i8" else "fp32"),
            "ms": round(ms, 5), "gflops": round(gflops, 1), "peak_tflops": peak,
            "frac_mfma_peak": round(gflops / 1e3 / peak, 4)}


def config_entry(w, ms):
    gflops = w.flops / (ms * 1e-3) / 1e9
    gbs = w.algorithmic_bytes / (ms * 1e-3) / 1e9
    return {"name": w.name, "kernel": "dconv_single_channel" if w.kind == "single" else "dconv_general",
            "shape": {"N": w.N, "C": w.C, "H": w.H, "W": w.W, "K": w.K, "F": w.F},
            "ms": round(ms, 5), "gflops": round(gflops, 1),
            "frac_fp32_peak": round(gflops / 1e3 / FP32_PEAK_TFLOPS, 4),
            "algorithmic_gbs": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}


def read_traffic(name):
    """HBM bytes per launch from the committed counter summary of this kernel/workload, if any."""
    p = ROOT / "profiles" / f"{name}_hbm_traffic.txt"
    if not p.exists():
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", p.read_text(), re.M)
    return float(m.group(1)) if m else None


def cpu_baseline(w, x, f):
    """The oracle as it stands, on a band of the headline workload, all host cores."""
    import numpy as np
    import oracle
    rows_out = w.Ho
    band = np.ascontiguousarray(x[:rows_out + w.F - 1])
    t0 = time.perf_counter()
    _, threads = oracle.single_channel(band, f, only32=True)
    dt = time.perf_counter() - t0
    flops = 2.0 * w.K * rows_out * w.Wo * w.F * w.F
    return {"value": round(flops / dt / 1e9, 3), "unit": "GFLOP/s", "cores": int(threads),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"{rows_out} of {w.Ho} output rows of the same image, all {w.K} filters"}


def oracle_sample(w, x, f, threads=0, budget_gflop=40.0):
    """Time the oracle on a bounded part of a configuration (a band of rows of the single image,
    or the first images of the batch), on `threads` host threads (0 = all)."""
    import numpy as np
    import oracle
    if w.kind == "single":
        per_row = 2.0 * w.K * w.Wo * w.F * w.F
        rows = int(max(1, min(w.Ho, budget_gflop * 1e9 // per_row)))
        band = np.ascontiguousarray(x[:rows + w.F - 1])
        t0 = time.perf_counter()
        _, used = oracle.single_channel(band, f, threads=threads, only32=True)
        dt = time.perf_counter() - t0
        flops, what = per_row * rows, f"{rows} of {w.Ho} output rows"
    else:
        per_img = w.flops / w.N
        n = int(max(1, min(w.N, budget_gflop * 1e9 // per_img)))
        t0 = time.perf_counter()
        _, _, used = oracle.general(np.ascontiguousarray(x[:n]), f, threads=threads)
        dt = time.perf_counter() - t0
        flops, what = per_img * n, f"{n} of {w.N} images"
    return {"gflops": round(flops / dt / 1e9, 2), "threads": int(used), "seconds": round(dt, 3),
            "sample": what}


def rotating_buffers_ms(w, steps):
    """Per-launch time of a small configuration with every launch on its own set of buffers
    (more than 512 MB in all), so that neither inputs nor outputs are served from a cache."""
    import torch
    import workloads as wl
    import paper_1705_10591_amd as dconv
    x, f = wl.make_inputs(w)
    per_set = 4 * (x.size + f.size + w.out_elems)
    nsets = int(600e6 // per_set) + 1
    xs = [torch.from_numpy(x).cuda() for _ in range(nsets)]
    fs = [torch.from_numpy(f).cuda() for _ in range(nsets)]
    outs = [torch.empty(w.out_shape(), dtype=torch.float32, device="cuda") for _ in range(nsets)]
    state = {"i": 0}

    def run():
        i = state["i"]
        state["i"] = (i + 1) % nsets
        if w.kind == "single":
            dconv.dconv_single_channel(xs[i], fs[i], out=outs[i])
        else:
            dconv.dconv_general(xs[i], fs[i], out=outs[i])
    ms, _ = time_launches(run, max(steps, 2 * nsets), nsets, warm_ms=60.0)
    return ms, nsets


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)
    peaks = None if (args.no_measured_peaks or args.only) else measured_peaks()
    import torch
    import workloads as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    allw = dict(wl.CONFIGS)
    allw.update({v.name: v for v in wl.S2_SWEEP.values()})
    allw.update(wl.PAPER_SWEEP)
    only, only_blocked = args.only, False
    if only and only.endswith("_blocked"):          # e.g. G3_bf16_blocked: the channel-blocked layout
        only, only_blocked = only[:-len("_blocked")], True
    if only and only.rsplit("_", 1)[-1] in ("f16", "bf16", "i8") and only.rsplit("_", 1)[0] in allw:
        # one of the short-data-type configurations on its own (for profiles): the same JSON shape
        wname, kind = only.rsplit("_", 1)
        w = allw[wname]
        run = make_half_runner(w, kind, blocked=only_blocked)
        ms, wall_ms = time_launches(run, args.steps, args.warmup, warm_ms=60.0)
        e = half_entry(w, kind, ms)
        if only_blocked:
            e["name"] += "_blocked"
        if args.copy_calibration:
            a = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
            b = torch.empty_like(a)
            for _ in range(3):
                b.copy_(a)
            torch.cuda.synchronize()
        print(json.dumps({
            "metric": "GFLOP/s (direct convolution with 16-bit or 8-bit inputs, per conv shape)",
            "value": e["gflops"], "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(wall_ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": kind, "data": "synthetic",
            "config": {"workload": f"{e['name']}: {e['kernel']} " + json.dumps(e["shape"]).replace('"', "")},
            "roofline": {"bound": "mfma", "achieved": round(e["gflops"] / 1e3, 3), "peak": e["peak_tflops"],
                         "unit": "TFLOP/s", "frac": e["frac_mfma_peak"], "kernel": e["kernel"],
                         "kernel_ms": round(ms, 5), "traffic": read_traffic(f"{e['kernel']}_{e['name']}")}}),
              flush=True)
        return
    head = allw[args.only] if args.only else wl.S2

    run, (x, f) = make_runner(head)
    ms, wall_ms = time_launches(run, args.steps, args.warmup, warm_ms=60.0)
    entry = config_entry(head, ms)

    single = head.kind == "single"
    # which roof bounds the workload: the one its time under that roof alone is longer for
    # (algorithmic bytes at the HBM peak against flops at the fp32 matrix-core peak); for the
    # single-channel configurations that is HBM up to 5x5 filters
    t_hbm = entry["algorithmic_gbs"] * ms / HBM_PEAK_GBS
    t_mfma = entry["gflops"] * ms / (FP32_PEAK_TFLOPS * 1e3)
    hbm_bound = t_hbm > t_mfma
    if hbm_bound:
        roof = {"bound": "hbm", "achieved": entry["algorithmic_gbs"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(entry["algorithmic_gbs"] / HBM_PEAK_GBS, 4)}
    else:
        # the few-filters kernels compute on the vector ALU: same published fp32 peak (it counts
        # the packed forms, which this build switches off: plain multiply-adds reach half of it)
        import paper_1705_10591_amd as dconv
        sh = entry["shape"]
        on_alu = dconv.tile_choice(single, sh["N"], sh["C"], sh["H"], sh["W"], sh["K"], sh["F"]) == dconv.CHOICE_FEW_FILTERS
        roof = {"bound": "alu" if on_alu else "mfma", "achieved": round(entry["gflops"] / 1e3, 3),
                "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(entry["gflops"] / 1e3 / FP32_PEAK_TFLOPS, 4)}
        if on_alu:
            roof["peak_plain_fma"] = FP32_PEAK_TFLOPS / 2
            roof["frac_plain_fma"] = round(entry["gflops"] / 1e3 / (FP32_PEAK_TFLOPS / 2), 4)
    roof["kernel"] = entry["kernel"]
    roof["kernel_ms"] = round(ms, 5)
    roof["traffic"] = read_traffic(f"{entry['kernel']}_{head.name}")
    roof["traffic_source"] = (f"profiles/{entry['kernel']}_{head.name}_hbm_traffic.txt (rocprofv3 counters of an "
                              "earlier run of the same command, not measured in this run)")
    if peaks:
        measured = peaks["hbm_fill_gbs"] if hbm_bound else peaks["fp32_mfma_tflops"]
        roof["peak_measured"] = measured
        roof["frac_measured"] = round(roof["achieved"] / measured, 4)
    add_measured(entry, peaks)

    result = {
        "metric": "GFLOP/s (fp32 direct convolution, per conv shape; % of fp32 peak and HBM GB/s alongside)",
        "value": entry["gflops"], "unit": "GFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{head.name}: {entry['kernel']} " + json.dumps(entry["shape"]).replace('"', "")},
        "roofline": roof,
    }
    if peaks:
        result["measured_peaks"] = peaks
    del run
    torch.cuda.empty_cache()

    if args.copy_calibration:
        n = 1 << 28                                   # 2^28 floats = 1 GiB read + 1 GiB written
        a = torch.ones(n, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()

    if not args.no_extra_configs and not args.only:
        per = [entry]
        order = ["S1", "S2_F3", "S2_F7", "S2_F9", "S2_F11", "G1", "G2", "G3"]
        for name in order:
            w = allw[name]
            r, (xw, fw) = make_runner(w)
            m, _ = time_launches(r, max(5, min(args.steps, 50)), max(2, min(args.warmup, 10)), warm_ms=60.0)
            e = add_measured(config_entry(w, m), peaks)
            if name in ("S1", "G2"):
                # the two launch-bound configurations: the same calls replayed from a HIP graph
                e["ms_graph_replay"] = round(graph_replay_ms(r), 5)
            del r
            torch.cuda.empty_cache()
            if name == "S1":
                # 4 MB of output fit the caches: also time it with every launch on fresh buffers
                e["ms_rotating_buffers"], e["rotating_sets"] = (lambda t: (round(t[0], 5), t[1]))(
                    rotating_buffers_ms(w, max(5, min(args.steps, 50))))
            if not args.no_cpu_baseline:
                # the oracle on a bounded part of the same configuration, all host threads
                # (one thread too for the two smallest), and what the whole would take over the GPU
                o = oracle_sample(w, xw, fw)
                e["oracle"] = o
                e["oracle_over_gpu_time"] = round((w.flops / (o["gflops"] * 1e9)) / (m * 1e-3), 1)
                if name in ("S1", "G2"):
                    e["oracle_one_thread"] = oracle_sample(w, xw, fw, threads=1, budget_gflop=2.0)
            per.append(e)
        result["per_config"] = per
        g = {e["name"]: e for e in per}
        result["roofline_general"] = {
            "bound": "mfma", "kernel": "dconv_general", "workload": "G3",
            "achieved": round(g["G3"]["gflops"] / 1e3, 3), "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": g["G3"]["frac_fp32_peak"], "traffic": read_traffic("dconv_general_G3"),
            "traffic_source": "profiles/dconv_general_G3_hbm_traffic.txt (earlier run)"}
        if peaks:
            result["roofline_general"]["peak_measured"] = peaks["fp32_mfma_tflops"]
            result["roofline_general"]["frac_measured"] = g["G3"]["frac_fp32_mfma_measured"]

    if not args.no_extra_configs and not args.only:
        # the next row of the scope: the same general-case shapes with fp16, bf16 and int8 inputs
        # (channels innermost), priced against the dense matrix-core peak of their type
        half = []
        for name in ("G2", "G3"):
            for kind in ("f16", "bf16", "i8"):
                r = make_half_runner(allw[name], kind)
                m, _ = time_launches(r, max(5, min(args.steps, 50)), max(2, min(args.warmup, 10)), warm_ms=60.0)
                half.append(half_entry(allw[name], kind, m))
                del r
                torch.cuda.empty_cache()
        # the same kernel fed from the channel-blocked layout (contiguous staging loads)
        r = make_half_runner(allw["G3"], "bf16", blocked=True)
        m, _ = time_launches(r, max(5, min(args.steps, 50)), max(2, min(args.warmup, 10)), warm_ms=60.0)
        e = half_entry(allw["G3"], "bf16", m)
        e["name"] += "_blocked"
        e["layout"] = "in[N][C/16][H][W][16], filt[K][C/16][F][F][16], out[N][K][Ho][Wo] fp32"
        half.append(e)
        del r
        torch.cuda.empty_cache()
        if peaks:
            for e in half:
                if e["name"].endswith("i8") or e["name"].endswith("i8_blocked"):
                    e["frac_int8_mfma_measured"] = round(e["gflops"] / 1e3 / peaks["int8_mfma_tops"], 4)
                else:
                    e["frac_bf16_mfma_measured"] = round(e["gflops"] / 1e3 / peaks["bf16_mfma_tflops"], 4)
        result["per_config_short_types"] = half
        best = max((e for e in half if e["name"].endswith("f16")), key=lambda e: e["gflops"])
        result["roofline_16bit"] = {"bound": "mfma", "kernel": best["kernel"], "workload": best["name"],
                                    "achieved": round(best["gflops"] / 1e3, 3), "peak": MFMA16_PEAK_TFLOPS,
                                    "unit": "TFLOP/s", "frac": best["frac_mfma_peak"],
                                    "traffic": read_traffic(f"{best['kernel']}_{best['name']}"),
                                    "traffic_source": f"profiles/{best['kernel']}_{best['name']}_hbm_traffic.txt (earlier run)"}
        if peaks:
            result["roofline_16bit"]["peak_measured"] = peaks["bf16_mfma_tflops"]
            result["roofline_16bit"]["frac_measured"] = round(best["gflops"] / 1e3 / peaks["bf16_mfma_tflops"], 4)

    if args.paper_sweep:
        sweep = []
        for name, w in wl.PAPER_SWEEP.items():
            r, _ = make_runner(w)
            m, _ = time_launches(r, max(5, min(args.steps, 50)), max(2, min(args.warmup, 10)), warm_ms=60.0)
            sweep.append(config_entry(w, m))
            del r
            torch.cuda.empty_cache()
        result["paper_sweep"] = sweep

    if not args.no_cpu_baseline and head.kind == "single":
        result["cpu_baseline"] = cpu_baseline(head, x, f)
    elif not args.no_cpu_baseline:
        import oracle
        import numpy as np
        n_img = 1
        t0 = time.perf_counter()
        _, _, thr = oracle.general(np.ascontiguousarray(x[:n_img]), f)
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": round(head.flops / head.N * n_img / dt / 1e9, 3),
                                  "unit": "GFLOP/s", "cores": int(thr), "kind": "oracle",
                                  "seconds": round(dt, 2), "sample": f"first {n_img} image(s) of the batch"}
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
