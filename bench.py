#!/usr/bin/env python3
"""Throughput of the optimizer hot path on one MI355X.

A step is one pass of the whole path over the workload: global gradient norm and
overflow flag (zi_grad_norm), then the fused AdamW update that reads that result
on the device (zi_adamw_step).  The default workload is the 1.3e9-element flat
HBM-resident state (fp32 p/m/v, bf16 gradients, bf16 copy out).

Prints ONE JSON line: the whole-job params/s, the roofline of the dominant kernel
(the fused update, timed with HIP events on the stream it runs on), the CPU
oracle timed on a bounded sample, and the streamed step's host-link figures.
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
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-streamed", action="store_true")
    ap.add_argument("--no-tensor-list", action="store_true", help="leave out the tensor-list figure (profiling runs)")
    ap.add_argument("--cpu-sample", type=int, default=1_300_000_000, help="elements the oracle is timed on")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="only run a plain device copy of 1 GiB five times (scales rocprofv3 byte counters)")
    ap.add_argument("--file-numel", type=int, default=1 << 28,
                    help="elements of the file-tier figure (three files of 4 bytes each; 0 = leave it out)")
    ap.add_argument("--streamed-numel", type=int, default=1 << 30,
                    help="elements of the host-resident state used for the streamed measurement")
    return ap.parse_args()


def resident(args, torch, zi, zs):
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    w = zs.workload(args.workload)
    n = args.numel or w["numel"][0]
    dt = w["lp_dtype"]
    spec = w["spec"]
    dev = torch.device("cuda:0")
    log(f"generating {args.workload}: {n} elements")
    p = torch.empty(n, dtype=torch.float32, device=dev)
    m = torch.empty(n, dtype=torch.float32, device=dev)
    v = torch.empty(n, dtype=torch.float32, device=dev)
    g = torch.empty(n, dtype=torch.int16, device=dev)
    lp = torch.zeros(n, dtype=torch.int16, device=dev)
    chunk = 1 << 26
    st32 = torch.empty(min(chunk, n), dtype=torch.float32, pin_memory=True)
    st16 = torch.empty(min(chunk, n), dtype=torch.int16, pin_memory=True)
    for lo in range(0, n, chunk):
        c = min(chunk, n - lo)
        for fill, out in ((spec.fill_p, p), (spec.fill_m, m), (spec.fill_v, v)):
            fill(st32, c, 0, lo)
            out[lo:lo + c].copy_(st32[:c])
        spec.fill_g(st16, c, 0, lo)
        g[lo:lo + c].copy_(st16[:c])
    del st32, st16

    cfg = zi.make_config(lr=w["lr"], beta1=w["beta1"], beta2=w["beta2"], eps=w["eps"],
                         weight_decay=w["weight_decay"], step=w["step"], loss_scale=w["loss_scale"],
                         max_grad_norm=w["max_grad_norm"])
    tl = zi.make_tensors([(p, m, v, g, lp, n)])
    d_norm = torch.zeros(3, dtype=torch.float64, device=dev)
    ws = torch.empty(zi.zi_norm_workspace_bytes(), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def one_step(ev=None):
        zi.zi_grad_norm(tl, dt, w["loss_scale"], d_norm, ws, stream=stream)
        if ev is not None:
            ev[0].record(stream)
        zi.zi_adamw_step(tl, dt, cfg, d_norm, stream=stream)
        if ev is not None:
            ev[1].record(stream)

    log(f"warmup {args.warmup}, timing {args.steps} steps")
    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True),
               torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        events[k][2].record(stream)
        one_step(events[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec_per_step = (t1 - t0) / args.steps
    k_ms = sum(e[0].elapsed_time(e[1]) for e in events) / args.steps       # fused update kernel
    n_ms = sum(e[2].elapsed_time(e[0]) for e in events) / args.steps       # norm pass (2 launches)
    flag = int(d_norm.cpu().numpy()[2:3].view("uint32")[0])
    if flag != 0:
        raise RuntimeError("synthetic gradients raised the overflow flag: the timed steps were skipped")

    # HBM bytes per launch from hardware counters (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a
    # copy kernel of known size): measured offline on this workload, recorded with its commands.
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "adamw_wide_kernel_c1_hbm_traffic.txt")
    if args.workload == "c1" and not args.numel and os.path.exists(tpath):
        for ln in open(tpath):
            if ln.startswith("traffic_bytes_per_launch"):
                traffic = int(ln.split("=")[1])
    achieved = BYTES_PER_ELEM_STEP * n / (k_ms * 1e-3) / 1e9

    # Practical ceilings of this device, same run, same buffers: a pure read, a 1:1 copy and an
    # in-place update with the fused step's access shape and no arithmetic.
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
        ceil[name + "_GBps"] = round(moved / (sorted(ts)[len(ts) // 2] * 1e-3) / 1e9, 1)
    # A ragged tensor list carved from the same buffers (one transformer layer at hidden size 8192: four
    # matrices of 67M-268M elements and eight vectors of 8K-32K), beside one flat tensor of the same length.
    tensor_list = None
    shapes = [k for _, k in zs.transformer_layer_shapes(8192)]
    if sum(shapes) <= n and not args.no_tensor_list:
        def timed_step(items):
            t_l = zi.make_tensors(items)
            ts = []
            for _ in range(6):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                zi.zi_grad_norm(t_l, dt, w["loss_scale"], d_norm, ws, stream=stream)
                a.record(stream)
                zi.zi_adamw_step(t_l, dt, cfg, d_norm, stream=stream)
                b.record(stream)
                b.synchronize()
                ts.append(a.elapsed_time(b))
            return sorted(ts[1:])[len(ts[1:]) // 2]
        items, o = [], 0
        for k in shapes:
            items.append((p[o:o + k], m[o:o + k], v[o:o + k], g[o:o + k], lp[o:o + k], k))
            o += k
        ms_list = timed_step(items)
        ms_flat = timed_step([(p[:o], m[:o], v[:o], g[:o], lp[:o], o)])
        tensor_list = dict(what=f"fused step over a list of {len(shapes)} tensors ({o} elements: one transformer layer "
                                "at hidden size 8192), beside one flat tensor of the same length",
                           list_GBps=round(BYTES_PER_ELEM_STEP * o / (ms_list * 1e-3) / 1e9, 1),
                           flat_GBps=round(BYTES_PER_ELEM_STEP * o / (ms_flat * 1e-3) / 1e9, 1),
                           list_over_flat=round(ms_flat / ms_list, 4))
    out = dict(
        n=n, sec_per_step=sec_per_step, tensor_list=tensor_list,
        roofline=dict(bound="hbm", kernel="adamw_wide_kernel", achieved=round(achieved, 1), peak=HBM_PEAK_GBS,
                      unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4), traffic=traffic,
                      bytes_per_launch=BYTES_PER_ELEM_STEP * n, kernel_ms=round(k_ms, 4)),
        norm=dict(kernel="sumsq_partial_kernel+norm_finalize_kernel", ms=round(n_ms, 4),
                  achieved_GBps=round(BYTES_PER_ELEM_NORM * n / (n_ms * 1e-3) / 1e9, 1),
                  frac_of_hbm_peak=round(BYTES_PER_ELEM_NORM * n / (n_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)),
        update_only_params_per_s=n / (k_ms * 1e-3),
        hbm_ceilings=dict(ceil, fused_step_frac_of_copy=round(achieved / ceil["copy_GBps"], 4),
                          norm_frac_of_read=round(BYTES_PER_ELEM_NORM * n / (n_ms * 1e-3) / 1e9 / ceil["read_GBps"], 4)),
        workload=f"{args.workload}: flat HBM-resident state of {n} elements (fp32 p/m/v, "
                 f"{'bf16' if dt == 0 else 'fp16'} gradients and copy), step {w['step']}; "
                 "step = gradient norm + overflow check + fused AdamW",
    )
    del p, m, v, g, lp
    torch.cuda.empty_cache()
    return out


def streamed(args, torch, zi, zs):
    """Host-link figures of the streamed step on a bounded slice of the host-resident workload."""
    w = zs.workload("c2")
    n = args.streamed_numel
    spec = w["spec"]
    dev = torch.device("cuda:0")
    log(f"streamed: pinning and generating 3 x {4 * n / 2**30:.1f} GiB of host state")
    hp = torch.empty(n, dtype=torch.float32, pin_memory=True)
    hm = torch.empty(n, dtype=torch.float32, pin_memory=True)
    hv = torch.empty(n, dtype=torch.float32, pin_memory=True)
    spec.fill_p(hp, n)
    spec.fill_m(hm, n)
    spec.fill_v(hv, n)
    g = torch.empty(n, dtype=torch.int16, device=dev)
    st16 = torch.empty(min(1 << 26, n), dtype=torch.int16, pin_memory=True)
    for lo in range(0, n, 1 << 26):
        c = min(1 << 26, n - lo)
        spec.fill_g(st16, c, 0, lo)
        g[lo:lo + c].copy_(st16[:c])
    lp = torch.zeros(n, dtype=torch.int16, device=dev)
    cfg = zi.make_config(lr=w["lr"], beta1=w["beta1"], beta2=w["beta2"], eps=w["eps"],
                         weight_decay=w["weight_decay"], step=w["step"])
    eng = zi.zi_engine_create(0, w["chunk_bytes"], w["n_slots"])
    tl = zi.make_tensors([(hp, hm, hv, g, lp, n)])
    try:
        probe_bytes = min(4 * n, 4 << 30)
        peaks = {}
        for mode, name in ((0, "h2d"), (1, "d2h"), (2, "bidir")):
            zi.zi_engine_link_probe(eng, hp, hm, probe_bytes, mode, 1)
            sec = min(zi.zi_engine_link_probe(eng, hp, hm, probe_bytes, mode, 1) for _ in range(3))
            peaks[name] = probe_bytes / sec / 1e9            # per direction
        spec.fill_m(hm, n)                                   # the probe wrote into hm
        torch.cuda.synchronize()
        # With and without the kernel, interleaved (the link's rate drifts by several percent between runs).
        times, copy_only = [], []
        zi.zi_adamw_step_streamed(eng, tl, w["lp_dtype"], cfg)      # warm-up
        for _ in range(5):
            zi.zi_engine_set_option(eng, zi.ZI_OPT_SKIP_KERNEL, 0)
            zi.zi_adamw_step_streamed(eng, tl, w["lp_dtype"], cfg)
            times.append(zi.zi_engine_last_stats(eng).seconds)
            zi.zi_engine_set_option(eng, zi.ZI_OPT_SKIP_KERNEL, 1)
            zi.zi_adamw_step_streamed(eng, tl, w["lp_dtype"], cfg)
            copy_only.append(zi.zi_engine_last_stats(eng).seconds)
        zi.zi_engine_set_option(eng, zi.ZI_OPT_SKIP_KERNEL, 0)
        st = zi.zi_engine_last_stats(eng)

        # Gradient-side offload: gradients and the low-precision copy in pinned host memory as well
        # (14 B/element each way), with the norm reduced from the host-resident gradients.
        log("streamed: gradients and copy offloaded too")
        hg = torch.empty(n, dtype=torch.int16, pin_memory=True)
        hg.copy_(g)
        hlp = torch.zeros(n, dtype=torch.int16, pin_memory=True)
        d_norm = torch.zeros(3, dtype=torch.float64, device=dev)
        ws = torch.empty(zi.zi_norm_workspace_bytes(), dtype=torch.uint8, device=dev)
        tl_off = zi.make_tensors([(hp, hm, hv, hg, hlp, n)])
        off_norm, off_step = [], []
        for _ in range(3):
            zi.zi_grad_norm_streamed(eng, tl_off, w["lp_dtype"], 1.0, d_norm, ws)
            off_norm.append(zi.zi_engine_last_stats(eng).seconds)
            zi.zi_adamw_step_streamed(eng, tl_off, w["lp_dtype"], cfg, d_norm)
            off_step.append(zi.zi_engine_last_stats(eng).seconds)
        del hg, hlp

        # The paper's own placement: the step on the host CPUs over host-resident state (no GPU involved);
        # beside it the link would carry only 2 B/element of gradients down and 2 B/element of copy up.
        log("streamed: host-CPU step on the same slice, for the crossover")
        hg2 = hp.numpy().view("uint16")[:n].copy()         # any 16-bit patterns of plausible magnitude
        hg2[:] = 0x3A00
        hlp2 = torch.zeros(n, dtype=torch.int16).numpy().view("uint16")
        tl_cpu = zi.make_tensors([(hp, hm, hv, hg2, hlp2, n)])
        ncores = min(os.cpu_count() or 1, 16)
        cpu_step = []
        for _ in range(3):
            t0c = time.perf_counter()
            zi.zi_host_adamw_step(tl_cpu, w["lp_dtype"], cfg, None, ncores)
            cpu_step.append(time.perf_counter() - t0c)
        del hg2, hlp2

        # State in ordinary (not page-locked) host memory, through a 6-slot pinned ring.
        log("streamed: ordinary host memory through the pinned ring")
        op, om, ov = hp.numpy().copy(), hm.numpy().copy(), hv.numpy().copy()
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_COPY_THREADS, 7)
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 6)
        tl_ring = zi.make_tensors([(op, om, ov, g, lp, n)])
        ring = []
        for _ in range(3):
            zi.zi_adamw_step_streamed(eng, tl_ring, w["lp_dtype"], cfg)
            ring.append(zi.zi_engine_last_stats(eng).seconds)
        del op, om, ov

        # State in files on the box's disk (direct I/O), through the same ring: the NVMe-tier figure.
        file_tier = file_tier_figures(args, zi, eng, spec, g, lp, w, cfg)
    finally:
        zi.zi_engine_destroy(eng)
    t = min(times)
    med = lambda xs: sorted(xs)[len(xs) // 2]
    per_dir = 12 * n / t / 1e9
    return dict(
        workload=f"slice of c2: {n} elements of fp32 p/m/v in pinned host memory, 64 MiB chunks, 3 slots",
        params_per_s=n / t, seconds=t, link_GBps_per_direction=round(per_dir, 2),
        measured_peak_GBps=dict((k, round(x, 2)) for k, x in peaks.items()),
        frac_of_bidir_peak=round(per_dir / peaks["bidir"], 4),
        hidden_ratio=round(med(times) / med(copy_only), 4), copy_only_seconds=med(copy_only),
        median_seconds=med(times),
        slot_uses=int(st.n_slot_uses),
        all_offloaded=dict(
            what="p, m, v, gradients and copy in pinned host memory: 14 B/element each way",
            step_GBps_per_direction=round(14 * n / min(off_step) / 1e9, 2),
            step_frac_of_bidir_peak=round(14 * n / min(off_step) / 1e9 / peaks["bidir"], 4),
            norm_GBps=round(2 * n / min(off_norm) / 1e9, 2),
            norm_frac_of_h2d_peak=round(2 * n / min(off_norm) / 1e9 / peaks["h2d"], 4)),
        host_cpu_step=dict(
            what=f"zi_host_adamw_step on the same slice, {ncores} threads (the paper's CPU-side placement); "
                 "reported for the crossover, never used as a fallback",
            params_per_s=n / min(cpu_step), host_memory_GBps=round(28 * n / min(cpu_step) / 1e9, 1)),
        ordinary_memory_ring=dict(
            what="p, m, v in ordinary host memory, 6-slot pinned ring, 7 copy threads per direction",
            GBps_per_direction=round(12 * n / min(ring) / 1e9, 2),
            frac_of_bidir_peak=round(12 * n / min(ring) / 1e9 / peaks["bidir"], 4)),
        file_tier=file_tier)


def file_tier_figures(args, zi, eng, spec, g, lp, w, cfg):
    """p, m, v in three files opened for direct I/O: the step's rate beside the storage's own two-way rate.
    The disk of the box is whatever it is (not an NVMe array); the fraction is the figure.  Any I/O
    problem (no space, no direct I/O on the file system) is reported, not fatal."""
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
                zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_COPY_THREADS, 16)
                zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 6)
                nbytes = 4 * n
                zi.zi_engine_file_probe(eng, -1, fds[3], nbytes)           # allocate the scratch file's blocks
                rd = nbytes / zi.zi_engine_file_probe(eng, fds[0], -1, nbytes) / 1e9
                wr = nbytes / zi.zi_engine_file_probe(eng, -1, fds[3], nbytes) / 1e9
                both = nbytes / zi.zi_engine_file_probe(eng, fds[1], fds[3], nbytes) / 1e9
                secs = []
                for _ in range(2):
                    zi.zi_adamw_step_files(eng, [(fds[0], fds[1], fds[2], 0, 0, 0, g, lp, n)], w["lp_dtype"], cfg)
                    secs.append(zi.zi_engine_last_stats(eng).seconds)
                rate = 12 * n / min(secs) / 1e9
                return dict(what=f"p, m, v of {n} elements in files (O_DIRECT), 6-slot pinned ring, 16 I/O threads per "
                                 "direction; storage rates from the engine's own probe on the same files",
                            storage_GBps=dict(read=round(rd, 2), write=round(wr, 2), both_each=round(both, 2)),
                            step_GBps_per_direction=round(rate, 2), frac_of_two_way_storage_rate=round(rate / both, 4),
                            params_per_s=n / min(secs))
            finally:
                for fd in fds:
                    os.close(fd)
    except (OSError, zi.ZiError) as e:
        return dict(error=f"{type(e).__name__}: {e}")


def cpu_baseline(args, zs):
    """The oracle as it stands, single thread, on the first `cpu_sample` elements of the workload."""
    import numpy as np
    import oracle
    w = zs.workload(args.workload)
    n = min(args.cpu_sample, args.numel or w["numel"][0])
    spec = w["spec"]
    log(f"cpu baseline: oracle on {n} elements")
    p = np.empty(n, np.float32); m = np.empty(n, np.float32); v = np.empty(n, np.float32)
    g = np.empty(n, np.uint16); lp = np.empty(n, np.uint16)
    spec.fill_p(p, n); spec.fill_m(m, n); spec.fill_v(v, n); spec.fill_g(g, n)
    cfg = oracle.config(lr=w["lr"], beta1=w["beta1"], beta2=w["beta2"], eps=w["eps"],
                        weight_decay=w["weight_decay"], step=w["step"], loss_scale=w["loss_scale"],
                        max_grad_norm=w["max_grad_norm"])
    t0 = time.perf_counter()
    sumsq, flag = oracle.grad_sumsq([g], w["lp_dtype"])
    oracle.adamw(p, m, v, g, lp, w["lp_dtype"], cfg, sumsq, flag)
    dt = time.perf_counter() - t0
    return dict(value=n / dt, unit="params/s", cores=1, kind="oracle",
                sample=f"first {n} elements of {args.workload} (gradient norm + AdamW, generation excluded), "
                       f"{dt:.1f} s on one of {os.cpu_count()} host cores")


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
                  hbm_ceilings=res["hbm_ceilings"], tensor_list=res["tensor_list"])
    if not args.no_streamed:
        extras["streamed"] = streamed(args, torch, zi, zs)
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
        "cpu_baseline": None if args.no_cpu_baseline else cpu_baseline(args, zs),
        "extras": extras,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
