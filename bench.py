#!/usr/bin/env python3
"""Benchmark: fwd + bwd_data + bwd_filter of the MobileNet-v1 depthwise stack (Table III's thirteen
layers), batch 128, fp32, once in NCHW and once in NHWC, on one MI355X.

A step is one pass of the whole hot path over the whole workload: for each layout, for each of
the 13 layers, dwconv_fwd, dwconv_bwd_filter (stage 1 + stage 2), dwconv_bwd_data through the
C ABI.  Every layer has its own device buffers (about 10 GB in all, far beyond the caches), so
each launch reads its operands from HBM.  Inputs are synthetic (seeded normal draws) and already
resident in HBM when the timed region starts.

Prints ONE JSON line.  `value` is algorithmic HBM bytes per second: for every pass
(|x| + |y|) * 4 bytes, divided by the wall time of the timed steps.
"""
import argparse
import json
import os
import sys
import time

PEAK_HBM_GBS = 8000.0
# fp32 vector peak: 256 compute units x 128 fp32 multiply-add lanes per clock x 2 flops x 2.4 GHz
PEAK_ALU_TFLOPS = 157.3
PEAK_MFMA_TFLOPS = {0: 157.3, 1: 2500.0}      # dense matrix-core peak by storage type: fp32, bf16
METRIC = "ms and HBM GB/s (% of peak) per fwd+bwd of MobileNet-v1 dw stack, batch 128"
PASS_NAMES = ("fwd", "bwd_data", "bwd_filter", "bwd")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2,
                    help="workload index 0..7 (default 2: the headline one; 5: MobileNet variant shapes; 6: group convolutions; "
                         "7: group convolutions in bf16)")
    ap.add_argument("--order", choices=["layer", "train"], default="layer",
                    help="launch order inside a step: layer by layer (fwd, bwd_filter, bwd_data of each), or as "
                         "a training step runs them (all forwards, then the backward passes from the last layer up)")
    ap.add_argument("--fused-bwd", action="store_true",
                    help="run the backward pass through dwconv_bwd (one call; a fused kernel where there is one, "
                         "which reads dy once: its algorithmic bytes are 2|x|+|y| instead of 2(|x|+|y|))")
    ap.add_argument("--side-stream", action="store_true",
                    help="enqueue each layer's filter gradient on a second stream, beside its input gradient")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and replay it for the timed steps (the library only enqueues "
                         "kernels on the stream it is given, so a step is capturable); takes the host's launch cost "
                         "out of the timed region")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true", help="skip the per-launch HIP-event pass")
    ap.add_argument("--report", action="store_true", help="print a per-layer table to stderr")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run two plain device copies of 1 GiB (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def build_ops(dw, wl, cfg, torch, order="layer", side=None, fused_bwd=False):
    """Allocate per-layer buffers and return the list of launches that make one step."""
    import ctypes
    ops = []
    lib = dw.load()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    stream2 = ctypes.c_void_p(side.cuda_stream) if side is not None else stream
    esz = 4 if cfg["dtype"] == wl.F32 else 2
    for layout in cfg["layouts"]:
        fwd_ops, bwd_ops = [], []
        # A layer that occurs `repeat` times in the stack gets several buffer sets, used in turn, so that at
        # least ~640 MB (more than the 256 MB Infinity Cache) is touched before a set comes round again: every
        # launch starts cold, as it does for the layers that occur once.
        expanded = []
        for li, (layer, repeat) in enumerate(cfg["layers"]):
            set_bytes = 2 * layer.pass_bytes(cfg["N"], esz)          # x, dx, y, dy
            nsets = max(1, min(repeat, -(-(640 << 20) // set_bytes)))
            expanded += [(li, layer, rep % nsets, rep < nsets) for rep in range(repeat)]
        made = {}
        for li, layer, si, fresh in expanded:
            repeat = 1
            if not fresh:
                f, bf, bd, b = made[(li, si)]
                if fused_bwd:
                    if order == "layer": ops += [f, b]
                    else: fwd_ops.append(f); bwd_ops.append((b,))
                elif order == "layer": ops += [f, bf, bd]
                else: fwd_ops.append(f); bwd_ops.append((bf, bd))
                continue
            x, w, dy = wl.make_inputs_device(layer, cfg["N"], layout, cfg["dtype"], seed=1000 * 7 + li + 131 * si)
            grouped = layer.cg > 1          # a group convolution: the gconv_* entry points
            if grouped:
                if fused_bwd:
                    raise SystemExit("bench.py: --fused-bwd has no group-convolution entry point")
                d = dw.group_desc(cfg["N"], layer.C, layer.H, layer.W, layer.K, layer.stride, layer.pad, layer.groups,
                                  layer.O, layout, cfg["dtype"])
                f_fwd, f_bd, f_bf = lib.gconv_fwd, lib.gconv_bwd_data, lib.gconv_bwd_filter
                ws_bytes, vname = dw.gconv_bwd_filter_workspace_bytes(d), dw.gconv_variant_name
            else:
                d = dw.desc(cfg["N"], layer.C, layer.H, layer.W, layer.K, layer.stride, layer.pad, layer.mult,
                            layout, cfg["dtype"])
                f_fwd, f_bd, f_bf = lib.dwconv_fwd, lib.dwconv_bwd_data, lib.dwconv_bwd_filter
                ws_bytes, vname = dw.bwd_filter_workspace_bytes(d), dw.variant_name
            y = torch.empty_like(dy); dx = torch.empty_like(x)
            dwt = torch.empty(w.shape, device="cuda", dtype=torch.float32)
            ws = torch.empty(max(ws_bytes, 16), device="cuda", dtype=torch.uint8)
            nbytes = layer.pass_bytes(cfg["N"], esz)
            # algorithmic flops of one pass: a multiply-add per tap (and per input channel of the group) and output element
            nflops = 2 * layer.K * layer.K * layer.cg * layer.y_elems(cfg["N"])
            common = dict(layer=layer.name, li=li, layout="NCHW" if layout == wl.NCHW else "NHWC",
                          bytes=nbytes, flops=nflops, repeat=repeat, stride=layer.stride, H=layer.H)
            # Pre-marshalled C-ABI calls (pointers and descriptor fixed once), so that the host enqueues
            # faster than the GPU drains and the timed region measures the kernels, not Python.
            dref = ctypes.byref(d)
            px, pw, pdy, py, pdx, pdw, pws = (ctypes.c_void_p(t.data_ptr()) for t in (x, w, dy, y, dx, dwt, ws))
            nws = ctypes.c_size_t(ws.numel())
            keep = (d, x, w, dy, y, dx, dwt, ws)

            def run_fwd(dref=dref, px=px, pw=pw, py=py, keep=keep, f_fwd=f_fwd):
                rc = f_fwd(dref, px, pw, py, stream)
                if rc: raise dw.DwconvError(rc, "dwconv_fwd")

            def run_bwd_data(dref=dref, pdy=pdy, pw=pw, pdx=pdx, keep=keep, f_bd=f_bd):
                rc = f_bd(dref, pdy, pw, pdx, stream)
                if rc: raise dw.DwconvError(rc, "dwconv_bwd_data")

            def run_bwd_filter(dref=dref, px=px, pdy=pdy, pdw=pdw, pws=pws, nws=nws, keep=keep, f_bf=f_bf):
                rc = f_bf(dref, px, pdy, pdw, pws, nws, stream)
                if rc: raise dw.DwconvError(rc, "dwconv_bwd_filter")

            def run_bwd_filter_side(dref=dref, px=px, pdy=pdy, pdw=pdw, pws=pws, nws=nws, keep=keep, f_bf=f_bf):
                rc = f_bf(dref, px, pdy, pdw, pws, nws, stream2)
                if rc: raise dw.DwconvError(rc, "dwconv_bwd_filter")

            # order within a layer: forward, filter gradient, input gradient.  The two backward passes
            # both read dy; run back to back, the second finds much of it in the 256 MB Infinity Cache.
            wsb = torch.empty(max(dw.bwd_workspace_bytes(d), 16), device="cuda", dtype=torch.uint8) if fused_bwd else ws
            pwsb, nwsb = ctypes.c_void_p(wsb.data_ptr()), ctypes.c_size_t(wsb.numel())

            def run_bwd(dref=dref, px=px, pdy=pdy, pw=pw, pdx=pdx, pdw=pdw, pwsb=pwsb, nwsb=nwsb, keep=(keep, wsb)):
                rc = lib.dwconv_bwd(dref, px, pdy, pw, pdx, pdw, pwsb, nwsb, stream)
                if rc: raise dw.DwconvError(rc, "dwconv_bwd")

            f = dict(common, which=0, variant=vname(d, 0), run=run_fwd)
            bf = dict(common, which=2, variant=vname(d, 2), run=run_bwd_filter, run_side=run_bwd_filter_side)
            bd = dict(common, which=1, variant=vname(d, 1), run=run_bwd_data)
            b = None
            if fused_bwd:
                vname = dw.variant_name(d, 3)
                # a fused kernel reads x and dy once and writes dx; without one the call runs the two passes
                bbytes = (2 * layer.x_elems(cfg["N"]) + layer.y_elems(cfg["N"])) * esz if vname != "separate" else 2 * nbytes
                b = dict(common, which=3, variant=vname, run=run_bwd, bytes=bbytes, flops=2 * nflops)
                if order == "layer":
                    ops += [f, b]
                else:
                    fwd_ops.append(f); bwd_ops.append((b,))
            elif order == "layer":
                ops += [f, bf, bd]
            else:
                fwd_ops.append(f); bwd_ops.append((bf, bd))
            made[(li, si)] = (f, bf, bd, b)
        if order == "train":
            ops += fwd_ops
            for grp in reversed(bwd_ops):
                ops += list(grp)
    return ops


def run_step(ops, main=None, side=None):
    """One step.  With a side stream the filter gradient of a layer is enqueued there once the layer's
    forward is done, and runs beside the input gradient (the two are independent in a training step);
    the step ends when both streams have drained into the main one."""
    if side is None:
        for op in ops:
            for _ in range(op["repeat"]):
                op["run"]()
        return
    for op in ops:
        for _ in range(op["repeat"]):
            if op["which"] == 2:
                side.wait_stream(main)
                op["run_side"]()
            else:
                op["run"]()
    main.wait_stream(side)


def time_kernels(ops, steps, torch):
    """Per-launch durations with HIP events on the launch stream (torch's current stream, the one the
    library is given), in the same cold-cache order as the timed steps.  An event pair with nothing
    between its two records already reads several microseconds on this stack; that empty-bracket
    time is measured live (median of 200) and subtracted.  Returns (ms per op: median over steps,
    empty-bracket ms)."""
    empties = []
    evs = []
    for _ in range(200):
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        a.record(); b.record(); evs.append((a, b))
    torch.cuda.synchronize()
    empties = sorted(a.elapsed_time(b) for a, b in evs)
    overhead = empties[len(empties) // 2]
    samples = [[] for _ in ops]
    for _ in range(steps):
        evs = []
        for op in ops:
            a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
            a.record(); op["run"](); b.record()
            evs.append((a, b))
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(evs):
            samples[i].append(a.elapsed_time(b))
    out = []
    for smp in samples:
        smp.sort()
        out.append(max(smp[len(smp) // 2] - overhead, 1e-4))
    return out, overhead


def stored_profile(workload, kernel_key):
    """What the committed rocprofv3 summaries of this workload say about `kernel_key`: HBM bytes per launch
    (FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy of known size) from profiles/hbm_traffic_<workload>.txt, and
    the average duration inside the profiled steps from profiles/kernel_stats_<workload>.txt (lines
    "traffic <key> <bytes>" and "instep <key> <launches> <avg us>"), with the commit that last changed each file so
    that a summary older than the kernels is visible."""
    import subprocess
    root = os.path.dirname(os.path.abspath(__file__))
    out = {"traffic": None, "traffic_file": None, "in_step_avg_us": None, "stats_file": None}
    for kind, tag, field in (("hbm_traffic", "traffic", "traffic"), ("kernel_stats", "instep", "in_step_avg_us")):
        rel = os.path.join("profiles", "%s_%s.txt" % (kind, workload))
        try:
            with open(os.path.join(root, rel)) as f:
                for line in f:
                    tok = line.split()
                    if len(tok) >= 3 and tok[0] == tag and tok[1] == kernel_key:
                        out[field] = int(float(tok[2])) if tag == "traffic" else float(tok[3])
        except OSError:
            continue
        try:
            h = subprocess.run(["git", "-C", root, "log", "-1", "--format=%h", "--", rel], capture_output=True,
                               text=True, timeout=10).stdout.strip()
        except (OSError, subprocess.SubprocessError):
            h = ""
        out["traffic_file" if tag == "traffic" else "stats_file"] = rel + ("@" + h if h else "")
    return out


def copy_ceiling(torch):
    """What a plain device-to-device copy reaches on this machine, as the achievable ceiling beside the 8 TB/s
    peak: 205.5 MB (the first layer's input at batch 128) copied between six rotating buffer pairs, so every
    copy starts cold like the benchmark's launches; bytes read + bytes written over the mean time of 24 copies."""
    n = 205520896 // 4
    bufs = [(torch.zeros(n, device="cuda"), torch.empty(n, device="cuda")) for _ in range(6)]
    for a, b in bufs:
        b.copy_(a)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 24
    e0.record()
    for i in range(reps):
        a, b = bufs[i % len(bufs)]
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    return {"GBps": round(2 * n * 4 / ms / 1e6, 1), "bytes_per_copy": 2 * n * 4, "what": "hipMemcpy device-to-device, cold, back to back"}


def cpu_baseline(wl, cfg):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: every layer, all three passes,
    every listed layout, batch capped at 128 (about ten seconds of oracle time on 16 threads)."""
    import numpy as np
    import oracle
    cores = min(oracle.threads_available(), os.cpu_count() or 1)
    Ns = min(cfg["N"], 128)
    total_bytes, total_s = 0, 0.0
    esz = 4 if cfg["dtype"] == wl.F32 else 2
    for layout in cfg["layouts"]:
        for li, (layer, repeat) in enumerate(cfg["layers"]):
            if layer.cg > 1:
                from oracle import gconv as orc
                x, w, dy = wl.make_group_inputs(Ns, layer.C, layer.O, layer.groups, layer.H, layer.W, layer.K,
                                                layer.stride, layer.pad, layout, cfg["dtype"], seed=li)
                kw = dict(K=layer.K, stride=layer.stride, pad=layer.pad, groups=layer.groups, O=layer.O, layout=layout,
                          nthreads=cores)
            else:
                orc = oracle
                x, w, dy = wl.make_inputs(layer, Ns, layout, cfg["dtype"], seed=li)
                kw = dict(K=layer.K, stride=layer.stride, pad=layer.pad, mult=layer.mult, layout=layout, nthreads=cores)
            x64, w64, dy64 = x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64)
            del x, dy
            t0 = time.perf_counter()
            orc.fwd(x64, w64, **kw)
            orc.bwd_data(dy64, w64, x_shape=x64.shape, **kw)
            orc.bwd_filter(x64, dy64, **kw)
            total_s += (time.perf_counter() - t0) * repeat
            total_bytes += 3 * layer.pass_bytes(Ns, esz) * repeat
            del x64, dy64
    # one thread, on one mid-sized layer (the oracle is the same loop nest; only the outer loop is split)
    mid = cfg["layers"][len(cfg["layers"]) // 2][0]
    Nm = min(cfg["N"], 32)
    if mid.cg > 1:
        from oracle import gconv as orc
        x, w, dy = wl.make_group_inputs(Nm, mid.C, mid.O, mid.groups, mid.H, mid.W, mid.K, mid.stride, mid.pad,
                                        cfg["layouts"][-1], cfg["dtype"], seed=99)
        kw = dict(K=mid.K, stride=mid.stride, pad=mid.pad, groups=mid.groups, O=mid.O, layout=cfg["layouts"][-1], nthreads=1)
    else:
        orc = oracle
        x, w, dy = wl.make_inputs(mid, Nm, cfg["layouts"][-1], cfg["dtype"], seed=99)
        kw = dict(K=mid.K, stride=mid.stride, pad=mid.pad, mult=mid.mult, layout=cfg["layouts"][-1], nthreads=1)
    x64, w64, dy64 = x.astype(np.float64), w.astype(np.float64), dy.astype(np.float64)
    t0 = time.perf_counter()
    orc.fwd(x64, w64, **kw); orc.bwd_data(dy64, w64, x_shape=x64.shape, **kw); orc.bwd_filter(x64, dy64, **kw)
    single = 3 * mid.pass_bytes(Nm, esz) / (time.perf_counter() - t0) / 1e9
    return dict(value=total_bytes / total_s / 1e9, unit="GB/s", cores=cores, kind="oracle",
                single_thread_GBps=round(single, 3), single_thread_sample="%s, batch %d, three passes" % (mid.name, Nm),
                sample="all layers of the workload, all three passes, %s, batch %d%s, fp64 loop nests, %d OpenMP "
                       "threads; timed: the oracle calls only (not input generation); algorithmic bytes counted at "
                       "the workload's element size" %
                       ("+".join("NCHW" if l == wl.NCHW else "NHWC" for l in cfg["layouts"]), Ns,
                        "" if Ns == cfg["N"] else " (reduced from %d)" % cfg["N"], cores),
                seconds=total_s)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus %d is not supported (no collectives, no "
              "sharding code exists here). Run with --gpus 1." % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_1803_09926_amd as dw
    from paper_1803_09926_amd import workloads as wl
    dw.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    cfg = wl.config(args.config)
    if args.calibrate_copy:
        # a plain copy of known size: 2^30 bytes read, 2^30 bytes written, per dispatch
        src = torch.zeros(1 << 28, device="cuda", dtype=torch.float32)
        dst = torch.empty_like(src)
        dst.copy_(src); dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.graph and args.side_stream:
        print("bench.py: --graph and --side-stream cannot be combined", file=sys.stderr)
        sys.exit(2)
    graph = None
    if args.graph:
        # the launches are bound to the stream that is current when they are built: build and capture on one stream
        cap = torch.cuda.Stream()
        torch.cuda.set_stream(cap)
    main_stream = torch.cuda.current_stream()
    side = torch.cuda.Stream() if args.side_stream else None
    ops = build_ops(dw, wl, cfg, torch, args.order, side, args.fused_bwd)
    step_bytes = sum(op["bytes"] * op["repeat"] for op in ops)
    if args.graph:
        run_step(ops, main_stream, side)           # one eager step first (loads the kernels)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=main_stream):
            run_step(ops, main_stream, side)
        step = graph.replay
    else:
        step = lambda: run_step(ops, main_stream, side)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    gbs = step_bytes / (dt / args.steps) / 1e9

    out = {
        "metric": METRIC if args.config == 2 else "ms and HBM GB/s (% of peak) per fwd+bwd of " + cfg["name"],
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if cfg["dtype"] == wl.F32 else "bf16", "data": "synthetic",
        "config": {"workload": cfg["name"], "batch": cfg["N"],
                   "layouts": ["NCHW" if l == wl.NCHW else "NHWC" for l in cfg["layouts"]],
                   "layers": len(cfg["layers"]), "passes": "fwd+bwd(one call)" if args.fused_bwd else "fwd+bwd_data+bwd_filter",
                   "step": "one fwd+bwd of the stack in every listed layout", "launch_order": args.order,
                   "launch": "hip graph replay" if args.graph else "eager"},
        "pct_of_peak_hbm": round(100.0 * gbs / PEAK_HBM_GBS, 2),
        "algorithmic_GB_per_step": round(step_bytes / 1e9, 4),
    }

    if not args.no_kernel_timing:
        kms, ev_overhead = time_kernels(ops, max(5, min(args.steps, 10)), torch)
        per_layout = {}
        by_variant = {}
        for op, ms in zip(ops, kms):
            per_layout.setdefault(op["layout"], {"ms": 0.0, "bytes": 0, "tail_ms": 0.0, "stride2_ms": 0.0,
                                                 "fwd_ms": 0.0, "bwd_data_ms": 0.0, "bwd_filter_ms": 0.0, "bwd_ms": 0.0})
            pl = per_layout[op["layout"]]
            pl["ms"] += ms * op["repeat"]; pl["bytes"] += op["bytes"] * op["repeat"]
            pl[PASS_NAMES[op["which"]] + "_ms"] += ms * op["repeat"]
            if op["H"] <= 14: pl["tail_ms"] += ms * op["repeat"]
            if op["stride"] == 2: pl["stride2_ms"] += ms * op["repeat"]
            key = PASS_NAMES[op["which"]] + ":" + op["variant"]
            v = by_variant.setdefault(key, {"ms": 0.0, "bytes": 0, "flops": 0, "launches": 0})
            v["ms"] += ms * op["repeat"]; v["bytes"] += op["bytes"] * op["repeat"]; v["launches"] += op["repeat"]
            v["flops"] += op["flops"] * op["repeat"]
        out["kernel_ms_per_stack"] = {k: {kk: round(vv, 4) for kk, vv in v.items() if kk != "bytes"} |
                                      {"GBps": round(v["bytes"] / v["ms"] / 1e6, 1)} for k, v in per_layout.items()}
        dom_key = max(by_variant, key=lambda k: by_variant[k]["ms"])
        dom = by_variant[dom_key]
        # The kernels of a step run back to back, and each lasts longer there than between two events (the event
        # records leave a gap in which the previous kernel's write-back drains).  In-step duration = bracketed
        # duration scaled by (wall time of a step) / (sum of all bracketed durations); the rocprofv3 kernel trace
        # of the same command (profiles/kernel_stats_<workload>.txt) gives the same figure within a few per cent.
        sum_bracketed = sum(ms * op["repeat"] for op, ms in zip(ops, kms))
        stretch = max(1.0, ms_per_step / sum_bracketed) if not args.side_stream else 1.0
        ms_in_step = dom["ms"] * stretch
        hbm_in_step = dom["bytes"] / ms_in_step / 1e6                    # GB/s
        hbm_bracketed = dom["bytes"] / dom["ms"] / 1e6
        alu_in_step = dom["flops"] / ms_in_step / 1e9                    # TFLOP/s
        ai = dom["flops"] / dom["bytes"]
        # which roofline binds: the one whose peak gives the longer minimum time for this kernel's bytes and flops
        # (a kernel that runs its contraction on the matrix cores is priced against their dense peak for its type)
        on_mfma = "mfma" in dom_key
        peak_flops = (PEAK_MFMA_TFLOPS[cfg["dtype"]] if on_mfma else PEAK_ALU_TFLOPS)
        alu_binds = dom["flops"] / (peak_flops * 1e12) > dom["bytes"] / (PEAK_HBM_GBS * 1e9)
        prof = stored_profile(cfg["name"], dom_key)
        roof = {"bound": ("mfma" if on_mfma else "alu") if alu_binds else "hbm", "kernel": dom_key,
                "achieved": round(alu_in_step if alu_binds else hbm_in_step, 1),
                "peak": peak_flops if alu_binds else PEAK_HBM_GBS, "unit": "TFLOP/s" if alu_binds else "GB/s",
                "frac": round(alu_in_step / peak_flops if alu_binds else hbm_in_step / PEAK_HBM_GBS, 4),
                "frac_is": "in-step: event-bracketed launch time x (step wall time / sum of bracketed times)",
                "frac_bracketed": round(hbm_bracketed / PEAK_HBM_GBS, 4),
                "in_step_stretch": round(stretch, 4),
                "traffic": prof["traffic"], "traffic_from": prof["traffic_file"],
                "launches_per_step": dom["launches"], "event_overhead_subtracted_ms": round(ev_overhead, 5),
                "avg_launch_ms": round(ms_in_step / dom["launches"], 5),
                "avg_launch_ms_bracketed": round(dom["ms"] / dom["launches"], 5),
                "algorithmic_bytes_per_launch": int(dom["bytes"] / dom["launches"]),
                "algorithmic_flops_per_launch": int(dom["flops"] / dom["launches"]),
                "flop_per_byte": round(ai, 2)}
        if prof["in_step_avg_us"]:
            # the same fraction from the committed kernel trace (average duration of this kernel inside the steps)
            roof["frac_profile"] = round(dom["bytes"] / dom["launches"] / (prof["in_step_avg_us"] * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)
            roof["profile_from"] = prof["stats_file"]
        if ai > 10.0:
            # near the ridge (157.3 TFLOP/s / 8 TB/s = 19.7 flop/B): both fractions
            roof["frac_hbm"] = round(hbm_in_step / PEAK_HBM_GBS, 4)
            roof["frac_mfma" if on_mfma else "frac_alu"] = round(alu_in_step / peak_flops, 4)
        out["roofline"] = roof
        # every kernel family of the step, against both rooflines (in-step durations)
        out["per_kernel"] = {k: {"launches": v["launches"], "in_step_ms": round(v["ms"] * stretch, 4),
                                 "frac_hbm": round(v["bytes"] / (v["ms"] * stretch) / 1e6 / PEAK_HBM_GBS, 4),
                                 ("frac_mfma" if "mfma" in k else "frac_alu"):
                                     round(v["flops"] / (v["ms"] * stretch) / 1e9 /
                                           (PEAK_MFMA_TFLOPS[cfg["dtype"]] if "mfma" in k else PEAK_ALU_TFLOPS), 4),
                                 "flop_per_byte": round(v["flops"] / v["bytes"], 2)}
                             for k, v in sorted(by_variant.items(), key=lambda kv: -kv[1]["ms"])}
        if args.report:
            print("%-34s %-5s %-10s %-28s %9s %9s %7s" % ("layer", "lay", "pass", "variant", "ms", "GB/s", "%peak"),
                  file=sys.stderr)
            for op, ms in zip(ops, kms):
                g = op["bytes"] / ms / 1e6
                print("%-34s %-5s %-10s %-28s %9.4f %9.1f %7.2f" % (op["layer"], op["layout"], PASS_NAMES[op["which"]],
                      op["variant"], ms, g, 100 * g / PEAK_HBM_GBS), file=sys.stderr)
            for k, v in sorted(by_variant.items(), key=lambda kv: -kv[1]["ms"]):
                print("variant %-44s launches %3d  ms %9.4f  GB/s %9.1f" % (k, v["launches"], v["ms"],
                      v["bytes"] / v["ms"] / 1e6), file=sys.stderr)
            out["per_op"] = [[op["layer"], op["layout"], PASS_NAMES[op["which"]], op["variant"], round(ms, 4)]
                             for op, ms in zip(ops, kms)]

    if not args.no_kernel_timing:
        out["copy_ceiling"] = copy_ceiling(torch)
        out["copy_ceiling"]["value_over_copy"] = round(gbs / out["copy_ceiling"]["GBps"], 3)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, cfg)
        out["cpu_baseline"]["value"] = round(out["cpu_baseline"]["value"], 3)
        out["cpu_baseline"]["seconds"] = round(out["cpu_baseline"]["seconds"], 2)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
