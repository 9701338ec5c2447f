#!/usr/bin/env python3
"""Throughput of the optimizer hot path on one MI355X.

A step is one pass of the whole path over the workload: global gradient norm and
overflow flag (zi_grad_norm), then the fused AdamW update that reads that result
on the device (zi_adamw_step).  The headline workload is c1, the 1.3e9-element flat
HBM-resident state (fp32 p/m/v, bf16 gradients, bf16 copy out).

Order of events: the first step on the seeded inputs is compared with the CPU oracle
over EVERY element (max and histogram of the ulp distance go into the line) before
anything is timed; then the timed steps; then the other workloads as extras (c0,
c3 fp16 with loss scale and clip, c4 tensor list resident and streamed, the c2 recipe
streamed from pinned host memory at the largest size that can be page-locked).

Prints ONE JSON line: whole-job params/s, the roofline of the dominant kernel (the
fused update, timed with HIP events on the stream it runs on), the oracle timed on
the host, the parity record, and the extras.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
BYTES_PER_ELEM_STEP = 28       # read p, m, v (4 B each) + g (2 B); write p, m, v + 2-byte copy
BYTES_PER_ELEM_NORM = 2
TRAFFIC_FILE = os.path.join("profiles", "adamw_wide_kernel_c1_hbm_traffic.txt")


def log(msg):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c1", choices=["c0", "c1", "c3"],
                    help="resident workload to time (c1 is the one the metric is quoted on)")
    ap.add_argument("--numel", type=int, default=0, help="override the element count (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="leave out the oracle (timing and parity)")
    ap.add_argument("--no-streamed", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="headline workload only (profiling runs)")
    ap.add_argument("--extras", default="c0,c3,c4,streamed", help="comma-separated extras to run (profiling runs)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="only run a plain device copy of 1 GiB five times (scales rocprofv3 byte counters)")
    ap.add_argument("--file-numel", type=int, default=1 << 28,
                    help="elements of the file-tier figure (three files of 4 bytes each; 0 = leave it out)")
    ap.add_argument("--streamed-numel", type=int, default=5_000_000_000,
                    help="elements of the host-resident state of the streamed measurement (falls back to 2^30 "
                         "if that much cannot be page-locked)")
    return ap.parse_args()


def median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


# ------------------------------------------------------------------------------------- helpers

def device_state(torch, spec, n, tensor=0):
    """p, m, v, g, lp on the device from the seeded recipe (through a pinned staging buffer)."""
    dev = torch.device("cuda:0")
    p = torch.empty(n, dtype=torch.float32, device=dev)
    m = torch.empty(n, dtype=torch.float32, device=dev)
    v = torch.empty(n, dtype=torch.float32, device=dev)
    g = torch.empty(n, dtype=torch.int16, device=dev)
    lp = torch.zeros(n, dtype=torch.int16, device=dev)
    chunk = 1 << 26
    st32 = torch.empty(min(chunk, max(n, 1)), dtype=torch.float32, pin_memory=True)
    st16 = torch.empty(min(chunk, max(n, 1)), dtype=torch.int16, pin_memory=True)
    for lo in range(0, n, chunk):
        c = min(chunk, n - lo)
        for fill, out in ((spec.fill_p, p), (spec.fill_m, m), (spec.fill_v, v)):
            fill(st32, c, tensor, lo)
            out[lo:lo + c].copy_(st32[:c])
        spec.fill_g(st16, c, tensor, lo)
        g[lo:lo + c].copy_(st16[:c])
    return p, m, v, g, lp


def host_state(np, spec, n, tensor=0):
    p = np.empty(n, np.float32); m = np.empty(n, np.float32); v = np.empty(n, np.float32)
    g = np.empty(n, np.uint16)
    spec.fill_p(p, n, tensor); spec.fill_m(m, n, tensor); spec.fill_v(v, n, tensor); spec.fill_g(g, n, tensor)
    return p, m, v, g


def ulp_histogram(torch, host_arr, dev_tensor, bits, block=1 << 27):
    """Distance between the order-preserving integer images of two arrays of bit patterns (host: the
    oracle's, device: the library's), over every element: [count at 0, 1, 2, more] and the maximum.
    +0 and -0 coincide.  The comparison itself runs on the device (the inputs are what is compared)."""
    import numpy as np
    n = host_arr.size
    it = torch.int32 if bits == 32 else torch.int16
    sign = 0x7FFFFFFF if bits == 32 else 0x7FFF
    hv = host_arr.view(np.int32 if bits == 32 else np.int16)
    stage = torch.empty(min(block, max(n, 1)), dtype=it, pin_memory=True)
    hist = [0, 0, 0, 0]
    worst = 0
    for lo in range(0, n, block):
        c = min(block, n - lo)
        stage.numpy()[:c] = hv[lo:lo + c]
        a = stage[:c].to("cuda:0").to(torch.int64)
        b = dev_tensor[lo:lo + c].view(it).to(torch.int64)
        a = torch.where(a < 0, -(a & sign), a)
        b = torch.where(b < 0, -(b & sign), b)
        d = (a - b).abs_()
        worst = max(worst, int(d.max())) if c else worst
        z = int((d == 0).sum()); o = int((d == 1).sum()); t = int((d == 2).sum())
        hist[0] += z; hist[1] += o; hist[2] += t; hist[3] += c - z - o - t
    return hist, worst


def parity_record(torch, zi, oracle, w, dev_arrays, host_in, what):
    """One step by the oracle on the host inputs (timed), compared with the device arrays element by element.
    Returns (parity dict, oracle seconds)."""
    import numpy as np
    p, m, v, g = host_in
    n = p.size
    dt = w["lp_dtype"]
    lp = np.zeros(n, np.uint16)
    cfg = oracle.config(lr=w["lr"], beta1=w["beta1"], beta2=w["beta2"], eps=w["eps"],
                        weight_decay=w["weight_decay"], step=w["step"], loss_scale=w["loss_scale"],
                        max_grad_norm=w["max_grad_norm"])
    t0 = time.perf_counter()
    sumsq, flag = oracle.grad_sumsq([g], dt)
    oracle.adamw(p, m, v, g, lp, dt, cfg, sumsq, flag)
    sec = time.perf_counter() - t0
    dp, dm, dv, dlp, d_norm = dev_arrays
    raw = d_norm.cpu().numpy()
    dsum, dflag = float(raw[0]), int(raw[2:3].view(np.uint32)[0])
    rec = dict(what=what, elements=n, found_inf=dict(oracle=int(flag), device=dflag),
               norm_rel=abs(dsum ** 0.5 - sumsq ** 0.5) / max(sumsq ** 0.5, 1e-300), max_ulp={}, hist={})
    for name, h, d, bits in (("p", p, dp, 32), ("m", m, dm, 32), ("v", v, dv, 32), ("lp", lp, dlp, 16)):
        hist, worst = ulp_histogram(torch, h, d, bits)
        rec["max_ulp"][name] = worst
        rec["hist"][name] = dict(zip(("0", "1", "2", ">2"), hist))
    rec["within_tolerance"] = bool(rec["max_ulp"]["p"] <= 2 and rec["max_ulp"]["m"] <= 2 and rec["max_ulp"]["v"] <= 2
                                   and rec["max_ulp"]["lp"] <= 1 and rec["norm_rel"] <= 1e-6
                                   and int(flag) == dflag)
    return rec, sec


def time_steps(torch, zi, tl, dt, loss_scale, cfg, d_norm, ws, stream, steps, warmup):
    """(seconds per whole step, [fused-kernel ms per step], [norm ms per step])."""
    for _ in range(warmup):
        zi.zi_grad_norm(tl, dt, loss_scale, d_norm, ws, stream=stream)
        zi.zi_adamw_step(tl, dt, cfg, d_norm, stream=stream)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    t0 = time.perf_counter()
    for k in range(steps):
        ev[k][0].record(stream)
        zi.zi_grad_norm(tl, dt, loss_scale, d_norm, ws, stream=stream)
        ev[k][1].record(stream)
        zi.zi_adamw_step(tl, dt, cfg, d_norm, stream=stream)
        ev[k][2].record(stream)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    return sec, [e[1].elapsed_time(e[2]) for e in ev], [e[0].elapsed_time(e[1]) for e in ev]


def stored_traffic(args):
    """HBM bytes per launch of the fused kernel from hardware counters.  Counters cannot be read from inside
    the process: the figure is the one recorded (with its rocprofv3 commands) for this workload."""
    path = os.path.join(ROOT, TRAFFIC_FILE)
    if args.workload == "c1" and not args.numel and os.path.exists(path):
        for ln in open(path):
            if ln.startswith("traffic_bytes_per_launch"):
                return int(ln.split("=")[1]), TRAFFIC_FILE + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, separate run)"
    return None, None


# ---------------------------------------------------------------------------- headline: resident

def resident(args, torch, zi, zs):
    import numpy as np
    w = zs.workload(args.workload)
    n = args.numel or w["numel"][0]
    dt, spec = w["lp_dtype"], w["spec"]
    dev = torch.device("cuda:0")
    log(f"generating {args.workload}: {n} elements")
    p, m, v, g, lp = device_state(torch, spec, n)
    cfg = zi.make_config(lr=w["lr"], beta1=w["beta1"], beta2=w["beta2"], eps=w["eps"],
                         weight_decay=w["weight_decay"], step=w["step"], loss_scale=w["loss_scale"],
                         max_grad_norm=w["max_grad_norm"])
    tl = zi.make_tensors([(p, m, v, g, lp, n)])
    d_norm = torch.zeros(4, dtype=torch.float64, device=dev)
    ws = torch.empty(zi.zi_norm_workspace_bytes(), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    # Parity first: one step on the seeded inputs, every element against the oracle.
    parity, cpu = None, None
    zi.zi_grad_norm(tl, dt, w["loss_scale"], d_norm, ws, stream=stream)
    zi.zi_adamw_step(tl, dt, cfg, d_norm, stream=stream)
    torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        import oracle
        log(f"oracle on all {n} elements of {args.workload} (host generation, one step, element-by-element comparison)")
        host_in = host_state(np, spec, n)
        parity, osec = parity_record(torch, zi, oracle, w, (p, m, v, lp, d_norm), host_in,
                                     f"{args.workload}: first step from the seeded inputs, every element of p, m, v and "
                                     "the copy against the oracle, before timing")
        del host_in
        cpu = dict(value=n / osec, unit="params/s", cores=1, kind="oracle",
                   sample=f"all {n} elements of {args.workload} (gradient norm + AdamW, generation excluded), "
                          f"{osec:.1f} s on one of {os.cpu_count()} host cores")
        log(f"parity: max ulp {parity['max_ulp']}, norm rel {parity['norm_rel']:.2e}")
        if not parity["within_tolerance"]:
            raise RuntimeError(f"parity failed before timing: {json.dumps(parity)}")

    log(f"warmup {args.warmup}, timing {args.steps} steps")
    sec_per_step, k_ms, n_ms = time_steps(torch, zi, tl, dt, w["loss_scale"], cfg, d_norm, ws, stream,
                                          args.steps, args.warmup)
    flag = int(d_norm.cpu().numpy()[2:3].view("uint32")[0])
    if flag != 0:
        raise RuntimeError("synthetic gradients raised the overflow flag: the timed steps were skipped")
    k_avg, n_avg = sum(k_ms) / len(k_ms), sum(n_ms) / len(n_ms)
    achieved = BYTES_PER_ELEM_STEP * n / (k_avg * 1e-3) / 1e9
    traffic, traffic_source = stored_traffic(args)

    # Practical ceilings of this device, same run, same buffers: a pure read, a 1:1 copy and an in-place
    # update of one array, launched in the shape that measured best for plain streams.
    ceil = {}
    nbytes = 4 * (n - n % 4)
    for mode, name, moved in ((0, "read", nbytes), (1, "copy", 2 * nbytes), (2, "update_in_place", 2 * nbytes)):
        ts = []
        for _ in range(7):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            zi.zi_hbm_probe(p, m, nbytes, mode, stream)
            b.record(stream)
            b.synchronize()
            ts.append(a.elapsed_time(b))
        ceil[name + "_GBps"] = round(moved / (median(ts) * 1e-3) / 1e9, 1)
    norm_gbps = BYTES_PER_ELEM_NORM * n / (n_avg * 1e-3) / 1e9
    out = dict(
        n=n, sec_per_step=sec_per_step, parity=parity, cpu=cpu,
        roofline=dict(bound="hbm", kernel="adamw_wide_kernel", achieved=round(achieved, 1), peak=HBM_PEAK_GBS,
                      unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4), traffic=traffic,
                      traffic_source=traffic_source, bytes_per_launch=BYTES_PER_ELEM_STEP * n,
                      kernel_ms=round(k_avg, 4), kernel_ms_min=round(min(k_ms), 4),
                      kernel_ms_median=round(median(k_ms), 4), kernel_ms_max=round(max(k_ms), 4),
                      frac_of_tuned_copy=round(achieved / ceil["copy_GBps"], 4)),
        norm=dict(kernel="sumsq_partial_kernel+norm_finalize_kernel", ms=round(n_avg, 4),
                  achieved_GBps=round(norm_gbps, 1), frac_of_hbm_peak=round(norm_gbps / HBM_PEAK_GBS, 4),
                  frac_of_tuned_read=round(norm_gbps / ceil["read_GBps"], 4)),
        update_only_params_per_s=n / (k_avg * 1e-3),
        hbm_ceilings=dict(ceil, what="zi_hbm_probe: single-wavefront groups, 4 KiB per wavefront, six wavefronts per "
                                     "CU, XCD-aware order; median of 7 launches over one 5.2 GB array"),
        workload=f"{args.workload}: flat HBM-resident state of {n} elements (fp32 p/m/v, "
                 f"{'bf16' if dt == 0 else 'fp16'} gradients and copy), step {w['step']}; "
                 "step = gradient norm + overflow check + fused AdamW",
    )
    del p, m, v, g, lp
    torch.cuda.empty_cache()
    return out


# ------------------------------------------------------------------------------ extras: c0, c3, c4

def extra_c0(args, torch, zi, zs):
    """The small parity workload: all 2^20 elements against the oracle, and its rate (it fits the last-level
    cache, so no roofline claim is made from it)."""
    import numpy as np
    import oracle
    w = zs.workload("c0")
    n, dt, spec = w["numel"][0], w["lp_dtype"], w["spec"]
    p, m, v, g, lp = device_state(torch, spec, n)
    cfg = zi.make_config(lr=w["lr"], beta1=w["beta1"], beta2=w["beta2"], eps=w["eps"],
                         weight_decay=w["weight_decay"], step=w["step"])
    tl = zi.make_tensors([(p, m, v, g, lp, n)])
    d_norm = torch.zeros(4, dtype=torch.float64, device="cuda:0")
    ws = torch.empty(zi.zi_norm_workspace_bytes(), dtype=torch.uint8, device="cuda:0")
    stream = torch.cuda.current_stream()
    zi.zi_grad_norm(tl, dt, 1.0, d_norm, ws, stream=stream)
    zi.zi_adamw_step(tl, dt, cfg, d_norm, stream=stream)
    torch.cuda.synchronize()
    best = None
    for _ in range(3):                                   # best of three for the small case
        host_in = host_state(np, spec, n)
        rec, osec = parity_record(torch, zi, oracle, w, (p, m, v, lp, d_norm), host_in, "c0: all elements")
        best = osec if best is None else min(best, osec)
    sec, k_ms, n_ms = time_steps(torch, zi, tl, dt, 1.0, cfg, d_norm, ws, stream, 50, 5)
    return dict(parity=rec, oracle_params_per_s=n / best, params_per_s=n / sec,
                kernel_us=round(1e3 * median(k_ms), 2), norm_us=round(1e3 * median(n_ms), 2),
                note="28 MiB of traffic: cache-resident and launch-bound, reported without a roofline claim")


def extra_c3(args, torch, zi, zs):
    """fp16 with loss scale 65536 at 2e9 elements.  Run A: +inf planted at a seeded index, the step must be
    skipped (every array bit-identical).  Run B: unscale, global norm, clip to 1.0, update; timed, and
    every element compared with the oracle."""
    import numpy as np
    import oracle
    w = zs.workload("c3")
    n, dt, spec = w["numel"][0], w["lp_dtype"], w["spec"]
    log(f"c3: generating {n} elements (fp16, loss scale {w['loss_scale']:.0f})")
    p, m, v, g, lp = device_state(torch, spec, n)
    cfg = zi.make_config(lr=w["lr"], beta1=w["beta1"], beta2=w["beta2"], eps=w["eps"],
                         weight_decay=w["weight_decay"], step=w["step"], loss_scale=w["loss_scale"],
                         max_grad_norm=w["max_grad_norm"])
    tl = zi.make_tensors([(p, m, v, g, lp, n)])
    d_norm = torch.zeros(4, dtype=torch.float64, device="cuda:0")
    ws = torch.empty(zi.zi_norm_workspace_bytes(), dtype=torch.uint8, device="cuda:0")
    stream = torch.cuda.current_stream()
    # run A
    j = zs.pick_index(spec.seed, 0x696E66, n)
    keep = int(g[j])
    g[j] = 0x7C00
    before = [x.clone() for x in (p, m, v, lp)]
    zi.zi_grad_norm(tl, dt, w["loss_scale"], d_norm, ws, stream=stream)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    zi.zi_adamw_step(tl, dt, cfg, d_norm, stream=stream)
    b.record(stream)
    torch.cuda.synchronize()
    flag_a = int(d_norm.cpu().numpy()[2:3].view("uint32")[0])
    same = all(torch.equal(x.view(torch.int32 if x.dtype == torch.float32 else torch.int16),
                           y.view(torch.int32 if y.dtype == torch.float32 else torch.int16))
               for x, y in zip(before, (p, m, v, lp)))
    skip_ms = a.elapsed_time(b)
    del before
    g[j] = keep
    # run B: parity on the first step, then timing
    zi.zi_grad_norm(tl, dt, w["loss_scale"], d_norm, ws, stream=stream)
    zi.zi_adamw_step(tl, dt, cfg, d_norm, stream=stream)
    torch.cuda.synchronize()
    log("c3: oracle on all 2e9 elements")
    host_in = host_state(np, spec, n)
    rec, osec = parity_record(torch, zi, oracle, w, (p, m, v, lp, d_norm), host_in,
                              "c3 run B: first step, every element against the oracle")
    del host_in
    raw = d_norm.cpu().numpy()
    norm = float(raw[0]) ** 0.5 / w["loss_scale"]
    sec, k_ms, n_ms = time_steps(torch, zi, tl, dt, w["loss_scale"], cfg, d_norm, ws, stream, 10, 2)
    k_avg, n_avg = sum(k_ms) / len(k_ms), sum(n_ms) / len(n_ms)
    ach = BYTES_PER_ELEM_STEP * n / (k_avg * 1e-3) / 1e9
    return dict(
        run_a=dict(inf_index=int(j), found_inf=flag_a, state_bit_identical=bool(same),
                   skipped_step_ms=round(skip_ms, 4)),
        run_b=dict(norm=norm, clip=min(1.0, w["max_grad_norm"] / (norm + 1e-6)), parity=rec,
                   params_per_s=n / sec, ms_per_step=sec * 1e3,
                   roofline=dict(bound="hbm", kernel="adamw_wide_kernel (fp16)", achieved=round(ach, 1),
                                 peak=HBM_PEAK_GBS, unit="GB/s", frac=round(ach / HBM_PEAK_GBS, 4),
                                 kernel_ms=round(k_avg, 4), kernel_ms_min=round(min(k_ms), 4)),
                   norm_ms=round(n_avg, 4), norm_GBps=round(2 * n / (n_avg * 1e-3) / 1e9, 1)),
        oracle_params_per_s=n / osec, oracle_seconds=round(osec, 2))


def link_peaks(zi, eng, src, dst, nbytes):
    """The link's own peaks, independent of the step's pacing: best over piece sizes and in-flight depths."""
    pieces = (16 << 20, 64 << 20, 192 << 20)
    table, best = {}, dict(h2d=0.0, d2h=0.0, bidir=0.0)
    for mode, name in ((0, "h2d"), (1, "d2h"), (2, "bidir")):
        for piece in pieces:
            for depth in (1, 2, 3, 0):
                if mode != 2 and depth in (1, 3):
                    continue                                 # one direction alone: pacing matters little
                sec = min(zi.zi_engine_link_probe(eng, src, dst, nbytes, mode, piece, depth) for _ in range(2))
                rate = nbytes / sec / 1e9
                table[f"{name}/piece{piece >> 20}MiB/depth{depth or 'inf'}"] = round(rate, 2)
                best[name] = max(best[name], rate)
    return best, table


def extra_c4(args, torch, zi, zs):
    """The ragged 48-tensor list (4 transformer layers at hidden size 8192, 3.2e9 elements): resident, and
    streamed from 144 separately pinned host arrays with a global clip."""
    import ctypes
    import numpy as np
    w = zs.workload("c4")
    numel, dt, spec = w["numel"], w["lp_dtype"], w["spec"]
    total = sum(numel)
    log(f"c4: {len(numel)} tensors, {total} elements: 144 pinned arrays + device gradients")
    cfg = zi.make_config(lr=w["lr"], beta1=w["beta1"], beta2=w["beta2"], eps=w["eps"],
                         weight_decay=w["weight_decay"], step=w["step"], loss_scale=w["loss_scale"],
                         max_grad_norm=w["max_grad_norm"])
    ptrs, host, grads, lps = [], [], [], []
    eng = None
    try:
        st16_ptr = zi.zi_pinned_alloc(2 * max(numel))
        ptrs.append(st16_ptr)
        st16 = np.ctypeslib.as_array((ctypes.c_int16 * max(numel)).from_address(st16_ptr))
        for i, n in enumerate(numel):
            arrs = []
            for fill in (spec.fill_p, spec.fill_m, spec.fill_v):
                ptr = zi.zi_pinned_alloc(4 * n)
                ptrs.append(ptr)
                a = np.ctypeslib.as_array((ctypes.c_float * n).from_address(ptr))
                fill(a, n, i)
                arrs.append(a)
            host.append(arrs)
            spec.fill_g(st16, n, i)
            grads.append(torch.from_numpy(st16[:n]).to("cuda:0"))
            lps.append(torch.zeros(n, dtype=torch.int16, device="cuda:0"))
        d_norm = torch.zeros(4, dtype=torch.float64, device="cuda:0")
        ws = torch.empty(zi.zi_norm_workspace_bytes(), dtype=torch.uint8, device="cuda:0")
        stream = torch.cuda.current_stream()
        tl_s = zi.make_tensors([(ptrs[1 + 3 * i], ptrs[2 + 3 * i], ptrs[3 + 3 * i], grads[i], lps[i], n)
                                for i, n in enumerate(numel)])
        eng = zi.zi_engine_create(0, w["chunk_bytes"], w["n_slots"])
        secs = []
        for _ in range(3):
            zi.zi_grad_norm(tl_s, dt, w["loss_scale"], d_norm, ws, stream=stream)
            zi.zi_adamw_step_streamed(eng, tl_s, dt, cfg, d_norm, stream)
            secs.append(zi.zi_engine_last_stats(eng).seconds)
        st = zi.zi_engine_last_stats(eng)
        probe = min(1 << 30, 4 * max(numel))
        big = max(range(len(numel)), key=lambda i: numel[i])
        peaks, _ = link_peaks(zi, eng, ptrs[1 + 3 * big], ptrs[2 + 3 * big], probe)
        zi.zi_engine_set_option(eng, zi.ZI_OPT_SKIP_KERNEL, 1)          # the same copies with the update removed
        zi.zi_adamw_step_streamed(eng, tl_s, dt, cfg, None, stream)
        peaks["bidir"] = max(peaks["bidir"], 12 * total / zi.zi_engine_last_stats(eng).seconds / 1e9)
        zi.zi_engine_set_option(eng, zi.ZI_OPT_SKIP_KERNEL, 0)
        raw = d_norm.cpu().numpy()
        streamed = dict(seconds=min(secs), GBps_per_direction=round(12 * total / min(secs) / 1e9, 2),
                        params_per_s=total / min(secs), slot_uses=int(st.n_slot_uses), copies=int(st.n_copies),
                        kernels=int(st.n_kernels),
                        frac_of_bidir_peak=round(12 * total / min(secs) / 1e9 / peaks["bidir"], 4),
                        frac_of_one_way_peak=round(12 * total / min(secs) / 1e9 / min(peaks["h2d"], peaks["d2h"]), 4),
                        grad_norm=float(raw[0]) ** 0.5)
        zi.zi_engine_destroy(eng)
        eng = None
        for ptr in ptrs:
            zi.zi_pinned_free(ptr)
        ptrs, host = [], []
        # the same list resident
        log("c4: the same list HBM-resident")
        res = []
        for i, n in enumerate(numel):
            p, m, v, _, _ = device_state(torch, spec, n, tensor=i)
            res.append((p, m, v))
        tl_r = zi.make_tensors([(res[i][0], res[i][1], res[i][2], grads[i], lps[i], n) for i, n in enumerate(numel)])
        sec, k_ms, n_ms = time_steps(torch, zi, tl_r, dt, w["loss_scale"], cfg, d_norm, ws, stream, 8, 2)
        k_avg = sum(k_ms) / len(k_ms)
        ach = BYTES_PER_ELEM_STEP * total / (k_avg * 1e-3) / 1e9
        resident = dict(params_per_s=total / sec, ms_per_step=sec * 1e3, update_ms=round(k_avg, 4),
                        update_GBps=round(ach, 1), update_frac_of_hbm_peak=round(ach / HBM_PEAK_GBS, 4),
                        norm_ms=round(sum(n_ms) / len(n_ms), 4),
                        launches="16 long tensors launched alone, 32 short ones share one launch")
        return dict(elements=total, tensors=len(numel), resident=resident, streamed_from_144_pinned_arrays=streamed)
    finally:
        if eng is not None:
            zi.zi_engine_destroy(eng)
        for ptr in ptrs:
            zi.zi_pinned_free(ptr)


# --------------------------------------------------------------------------- extras: host-resident

def streamed(args, torch, zi, zs):
    """The c2 recipe (fp32 p/m/v in pinned host memory, bf16 gradients and copy in HBM, 64 MiB chunks, three
    slots) at the largest size that can be page-locked, with the link's independent peaks beside it."""
    import numpy as np
    w = zs.workload("c2")
    spec = w["spec"]
    dev = torch.device("cuda:0")
    # The library's allocator is used for the big page-locked blocks: the tensor library's pinned allocator
    # rounds sizes up to powers of two and keeps freed blocks.
    import ctypes
    held = []

    def pinned_f32(count):
        ptr = zi.zi_pinned_alloc(4 * count)
        held.append(ptr)
        return torch.from_numpy(np.ctypeslib.as_array((ctypes.c_float * count).from_address(ptr)))

    hp = hm = hv = None
    for n in (args.streamed_numel, 4_000_000_000, 1 << 30):
        try:
            log(f"streamed: pinning 3 x {4 * n / 2**30:.1f} GiB of host state")
            hp, hm, hv = pinned_f32(n), pinned_f32(n), pinned_f32(n)
            break
        except zi.ZiError as e:
            log(f"streamed: {n} elements cannot be page-locked here ({e.message})")
            hp = hm = hv = None
            while held:
                zi.zi_pinned_free(held.pop())
    if hp is None:
        return dict(error="no page-locked memory for the host-resident state")
    piece = 1 << 30
    for lo in range(0, n, piece):
        c = min(piece, n - lo)
        spec.fill_p(hp[lo:lo + c], c, 0, lo)
        spec.fill_m(hm[lo:lo + c], c, 0, lo)
        spec.fill_v(hv[lo:lo + c], c, 0, lo)
    g = torch.empty(n, dtype=torch.int16, device=dev)
    st16 = torch.empty(min(1 << 26, n), dtype=torch.int16, pin_memory=True)
    for lo in range(0, n, 1 << 26):
        c = min(1 << 26, n - lo)
        spec.fill_g(st16, c, 0, lo)
        g[lo:lo + c].copy_(st16[:c])
    del st16
    lp = torch.zeros(n, dtype=torch.int16, device=dev)
    cfg = zi.make_config(lr=w["lr"], beta1=w["beta1"], beta2=w["beta2"], eps=w["eps"],
                         weight_decay=w["weight_decay"], step=w["step"])
    eng = zi.zi_engine_create(0, w["chunk_bytes"], w["n_slots"])
    tl = zi.make_tensors([(hp, hm, hv, g, lp, n)])
    try:
        log("streamed: link peaks (piece size x in-flight depth sweep)")
        scratch = zi.zi_pinned_alloc(2 << 30)                   # landing area of the device-to-host pieces
        try:
            peaks, table = link_peaks(zi, eng, hp, scratch, 2 << 30)
        finally:
            zi.zi_pinned_free(scratch)
        # With and without the kernel, interleaved (the link's rate drifts by several percent between runs).
        times, copy_only = [], []
        zi.zi_adamw_step_streamed(eng, tl, w["lp_dtype"], cfg)      # warm-up
        for _ in range(3):
            zi.zi_engine_set_option(eng, zi.ZI_OPT_SKIP_KERNEL, 0)
            zi.zi_adamw_step_streamed(eng, tl, w["lp_dtype"], cfg)
            times.append(zi.zi_engine_last_stats(eng).seconds)
            zi.zi_engine_set_option(eng, zi.ZI_OPT_SKIP_KERNEL, 1)
            zi.zi_adamw_step_streamed(eng, tl, w["lp_dtype"], cfg)
            copy_only.append(zi.zi_engine_last_stats(eng).seconds)
        zi.zi_engine_set_option(eng, zi.ZI_OPT_SKIP_KERNEL, 0)
        st = zi.zi_engine_last_stats(eng)
        t = min(times)
        per_dir = 12 * n / t / 1e9
        # The engine's own copy pattern with the update removed is one more way of driving the link: it
        # belongs to the sweep, so the two-way peak is the best rate any pure-copy pattern reached.
        table["bidir/engine pacing, update removed"] = round(12 * n / min(copy_only) / 1e9, 2)
        peaks["bidir"] = max(peaks["bidir"], 12 * n / min(copy_only) / 1e9)
        out = dict(
            workload=f"c2 recipe at {n} elements ({12 * n / 1e9:.0f} GB of fp32 p/m/v in pinned host memory; the "
                     "8e9-element original needs 96 GB page-locked, beyond this host's limit), 64 MiB chunks, 3 slots",
            params_per_s=n / t, seconds=t, link_GBps_per_direction=round(per_dir, 2),
            measured_peak_GBps=dict((k, round(x, 2)) for k, x in peaks.items()),
            peak_sweep_GBps=table,
            frac_of_bidir_peak=round(per_dir / peaks["bidir"], 4),
            frac_of_one_way_peak=round(per_dir / min(peaks["h2d"], peaks["d2h"]), 4),
            target="streamed step >= 0.85 of the measured pinned-copy peak: quoted against the best two-way rate "
                   "of the sweep (both directions busy, as in the step); the one-way figure is beside it",
            hidden_ratio=round(median(times) / median(copy_only), 4), copy_only_seconds=median(copy_only),
            median_seconds=median(times), slot_uses=int(st.n_slot_uses))

        # Everything below runs on a 2^30-element slice of the same state.
        ns = min(n, 1 << 30)
        tls = zi.make_tensors([(hp, hm, hv, g, lp, ns)])
        zi.zi_adamw_step_streamed(eng, tls, w["lp_dtype"], cfg)
        gpu_slice = []
        for _ in range(3):
            zi.zi_adamw_step_streamed(eng, tls, w["lp_dtype"], cfg)
            gpu_slice.append(zi.zi_engine_last_stats(eng).seconds)

        # Gradient-side offload: gradients and the low-precision copy in pinned host memory as well
        # (14 B/element each way), with the norm reduced from the host-resident gradients; and the
        # offload of freshly produced gradient partitions beside a producer that keeps running.
        log("streamed: gradients and copy offloaded too")
        hg = zi.zi_pinned_alloc(2 * ns)
        hlp = zi.zi_pinned_alloc(2 * ns)
        d_norm = torch.zeros(4, dtype=torch.float64, device=dev)
        ws = torch.empty(zi.zi_norm_workspace_bytes(), dtype=torch.uint8, device=dev)
        producer = torch.cuda.Stream()
        part = 1 << 26                                          # 64 Mi elements = 128 MiB per partition
        t0 = time.perf_counter()
        for lo in range(0, ns, part):
            c = min(part, ns - lo)
            zi.zi_grad_offload(eng, g[lo:], hg + 2 * lo, 2 * c, producer)
        t_issue = time.perf_counter() - t0
        zi.zi_grad_offload_wait(eng)
        t_off = time.perf_counter() - t0
        tl_off = zi.make_tensors([(hp, hm, hv, hg, hlp, ns)])
        off_norm, off_step = [], []
        for _ in range(3):
            zi.zi_grad_norm_streamed(eng, tl_off, w["lp_dtype"], 1.0, d_norm, ws)
            off_norm.append(zi.zi_engine_last_stats(eng).seconds)
            zi.zi_adamw_step_streamed(eng, tl_off, w["lp_dtype"], cfg, d_norm)
            off_step.append(zi.zi_engine_last_stats(eng).seconds)
        out["all_offloaded"] = dict(
            what=f"{ns} elements; p, m, v, gradients and copy in pinned host memory: 14 B/element each way",
            step_GBps_per_direction=round(14 * ns / min(off_step) / 1e9, 2),
            step_frac_of_bidir_peak=round(14 * ns / min(off_step) / 1e9 / peaks["bidir"], 4),
            norm_GBps=round(2 * ns / min(off_norm) / 1e9, 2),
            norm_frac_of_h2d_peak=round(2 * ns / min(off_norm) / 1e9 / peaks["h2d"], 4),
            grad_offload=dict(what="zi_grad_offload of the gradients in 128 MiB partitions",
                              issue_us_per_call=round(1e6 * t_issue / max(1, (ns + part - 1) // part), 1),
                              GBps=round(2 * ns / t_off / 1e9, 2),
                              frac_of_d2h_peak=round(2 * ns / t_off / 1e9 / peaks["d2h"], 4)))
        zi.zi_pinned_free(hg)
        zi.zi_pinned_free(hlp)

        # The paper's own placement, complete: the step on the host CPUs over the host-resident state,
        # gradients fetched from the device and the copy shipped back (2 + 2 B/element over the link),
        # beside the GPU placement of the same slice (12 + 12 B/element over the link).
        log("streamed: CPU placement (zi_adamw_step_cpu) beside the GPU placement, for the crossover")
        ncores = min(os.cpu_count() or 1, 16)
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 6)
        cpu_step = []
        for _ in range(4):
            zi.zi_adamw_step_cpu(eng, tls, w["lp_dtype"], cfg, None, ncores)
            cpu_step.append(zi.zi_engine_last_stats(eng).seconds)
        cpu_step = cpu_step[1:]
        hg2 = np.full(ns, 0x3A00, np.uint16)
        hlp2 = np.zeros(ns, np.uint16)
        tl_cpu = zi.make_tensors([(hp, hm, hv, hg2, hlp2, ns)])
        bare = []
        for _ in range(3):
            t0c = time.perf_counter()
            zi.zi_host_adamw_step(tl_cpu, w["lp_dtype"], cfg, None, ncores)
            bare.append(time.perf_counter() - t0c)
        del hg2, hlp2
        out["placement_crossover"] = dict(
            what=f"{ns} elements of host-resident fp32 state, gradients and copy in HBM; two complete placements of "
                 "the step",
            gpu_placement=dict(call="zi_adamw_step_streamed", link_bytes_per_element="12 down + 12 up",
                               params_per_s=ns / min(gpu_slice)),
            cpu_placement=dict(call=f"zi_adamw_step_cpu, {ncores} threads", link_bytes_per_element="2 down + 2 up",
                               params_per_s=ns / min(cpu_step), host_memory_GBps=round(28 * ns / min(cpu_step) / 1e9, 1),
                               bare_host_loop_params_per_s=ns / min(bare),
                               frac_of_bare_host_loop=round(min(bare) / min(cpu_step), 4)),
            cpu_over_gpu=round(min(gpu_slice) / min(cpu_step), 3))

        # State in ordinary (not page-locked) host memory, through a 6-slot pinned ring.
        log("streamed: ordinary host memory through the pinned ring")
        op, om, ov = hp[:ns].numpy().copy(), hm[:ns].numpy().copy(), hv[:ns].numpy().copy()
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_COPY_THREADS, 7)
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 6)
        tl_ring = zi.make_tensors([(op, om, ov, g, lp, ns)])
        ring = []
        for _ in range(3):
            zi.zi_adamw_step_streamed(eng, tl_ring, w["lp_dtype"], cfg)
            ring.append(zi.zi_engine_last_stats(eng).seconds)
        del op, om, ov
        out["ordinary_memory_ring"] = dict(
            what=f"{ns} elements; p, m, v in ordinary host memory, 6-slot pinned ring, 7 copy threads per direction",
            GBps_per_direction=round(12 * ns / min(ring) / 1e9, 2),
            frac_of_bidir_peak=round(12 * ns / min(ring) / 1e9 / peaks["bidir"], 4))

        # State in files on the box's disk (direct I/O), through the same ring: the NVMe-tier figure.
        out["file_tier"] = file_tier_figures(args, zi, eng, spec, g, lp, w, cfg)
        return out
    finally:
        zi.zi_engine_destroy(eng)
        del hp, hm, hv
        while held:
            zi.zi_pinned_free(held.pop())


def file_tier_figures(args, zi, eng, spec, g, lp, w, cfg):
    """p, m, v in three files opened for direct I/O: the step's rate beside the storage's own two-way rate
    (best over the number of requests in flight).  The disk of the box is whatever it is (not an NVMe array);
    the fraction is the figure.  Any I/O problem (no space, no direct I/O on the file system) is reported,
    not fatal."""
    import tempfile
    import numpy as np
    n = min(args.file_numel, g.numel())
    if n <= 0:
        return None
    n -= n % 1024                                   # 4096-byte multiple per array for the probe
    log(f"streamed: file tier, 3 x {4 * n / 2**30:.1f} GiB in {tempfile.gettempdir()}")
    fds = []
    try:
        with tempfile.TemporaryDirectory() as tmp:
            try:
                buf = np.empty(min(n, 1 << 26), np.float32)
                paths = [os.path.join(tmp, k + ".bin") for k in "pmv"]
                for path, fill in zip(paths, (spec.fill_p, spec.fill_m, spec.fill_v)):
                    with open(path, "wb") as f:
                        for lo in range(0, n, buf.size):
                            c = min(buf.size, n - lo)
                            fill(buf, c, 0, lo)
                            f.write(buf[:c].tobytes())
                os.sync()
                fds = [os.open(p, os.O_RDWR | os.O_DIRECT) for p in paths]
                fds.append(os.open(os.path.join(tmp, "scratch.bin"), os.O_RDWR | os.O_CREAT | os.O_DIRECT, 0o600))
                nbytes = 4 * n
                sweep, best_both, best_threads = {}, 0.0, 16
                for threads in (8, 16, 32, 64):
                    zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_COPY_THREADS, threads)
                    zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 6)
                    if not sweep:
                        zi.zi_engine_file_probe(eng, -1, fds[3], nbytes)       # allocate the scratch file's blocks
                    rd = nbytes / zi.zi_engine_file_probe(eng, fds[0], -1, nbytes) / 1e9
                    wr = nbytes / zi.zi_engine_file_probe(eng, -1, fds[3], nbytes) / 1e9
                    both = max(nbytes / zi.zi_engine_file_probe(eng, fds[1], fds[3], nbytes) / 1e9 for _ in range(2))
                    sweep[f"{threads}+{threads} requests"] = dict(read=round(rd, 2), write=round(wr, 2),
                                                                 both_each=round(both, 2))
                    if both > best_both:
                        best_both, best_threads = both, threads
                zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_COPY_THREADS, best_threads)
                zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 6)
                secs = []
                for _ in range(2):
                    zi.zi_adamw_step_files(eng, [(fds[0], fds[1], fds[2], 0, 0, 0, g, lp, n)], w["lp_dtype"], cfg)
                    secs.append(zi.zi_engine_last_stats(eng).seconds)
                rate = 12 * n / min(secs) / 1e9
                # the probe once more, after the step (the disk's rate drifts): the peak is the best seen
                again = max(nbytes / zi.zi_engine_file_probe(eng, fds[1], fds[3], nbytes) / 1e9 for _ in range(3))
                sweep[f"{best_threads}+{best_threads} requests, after the step (best of 3)"] = dict(both_each=round(again, 2))
                best_both = max(best_both, again)
                return dict(what=f"p, m, v of {n} elements in files (O_DIRECT), 6-slot pinned ring; the step runs "
                                 f"with {best_threads}+{best_threads} requests in flight, the count that gave the "
                                 "storage's best two-way rate in the sweep",
                            storage_GBps_by_requests_in_flight=sweep, storage_two_way_peak_GBps=round(best_both, 2),
                            step_GBps_per_direction=round(rate, 2),
                            frac_of_two_way_storage_peak=round(rate / best_both, 4),
                            note="a virtual disk whose rate drifts by several percent between runs; the peak is the best "
                                 "two-way rate any probe reached before or after the step",
                            params_per_s=n / min(secs))
            finally:
                for fd in fds:
                    os.close(fd)
    except (OSError, zi.ZiError) as e:
        return dict(error=f"{type(e).__name__}: {e}")


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no sharding and no collectives; run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback exists)", file=sys.stderr)
        sys.exit(2)
    if args.pmc_calibration:
        # A copy kernel of known size: reads 2^30 bytes and writes 2^30 bytes per launch.
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "5 device copies", "bytes_read_per_launch": 1 << 30,
                          "bytes_written_per_launch": 1 << 30}), flush=True)
        return
    import paper_2104_07857_amd as zi
    import zi_synth as zs
    zi.lib()

    res = resident(args, torch, zi, zs)
    extras = dict(update_only_params_per_s=res["update_only_params_per_s"], norm=res["norm"],
                  hbm_ceilings=res["hbm_ceilings"])
    if not args.no_extras:
        def attempt(name, fn):
            try:
                extras[name] = fn(args, torch, zi, zs)
            except Exception as e:                       # an extra never costs the headline line
                extras[name] = dict(error=f"{type(e).__name__}: {e}")
                log(f"{name} failed: {e}")
            torch.cuda.empty_cache()
        want = set(args.extras.split(","))
        if not args.no_cpu_baseline and "c0" in want:
            attempt("c0", extra_c0)
        if not args.no_cpu_baseline and "c3" in want:
            attempt("c3", extra_c3)
        if "c4" in want:
            attempt("c4", extra_c4)
        if not args.no_streamed and "streamed" in want:
            attempt("streamed", streamed)
    line = {
        "metric": "AdamW step params/s + % HBM peak (resident); % host-link BW (streamed)",
        "value": res["n"] / res["sec_per_step"],
        "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["sec_per_step"] * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": res["workload"]},
        "roofline": res["roofline"],
        "cpu_baseline": res["cpu"],
        "parity": res["parity"],
        "extras": extras,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
