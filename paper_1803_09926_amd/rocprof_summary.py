"""Turn rocprofv3 CSV output of `bench.py` into the short text summaries kept under profiles/.

Usage:
  python -m paper_1803_09926_amd.rocprof_summary stats   <dir with *_kernel_stats.csv> [workload index of bench.py --config [fused]]
  python -m paper_1803_09926_amd.rocprof_summary traffic <FETCH_SIZE dir> <WRITE_SIZE dir> [workload index]
  python -m paper_1803_09926_amd.rocprof_summary pmc     <dir of a --pmc run> [substring of the kernel names to keep]

`traffic` expects both runs to contain bench.py's --calibrate-copy dispatches (a plain device copy
of 2^30 bytes): each counter is scaled so that the copy reads (writes) exactly 2^30 bytes.
`fused` after the workload index: the trace is of `bench.py --fused-bwd`.
Output goes to stdout.
"""
import csv
import glob
import os
import re
import sys

# bench.py's "<pass>:<variant>" keys -> the kernel(s) that implement them (regex on the demangled name)
VARIANT_KERNELS = {
    # k_nhwc_s1<T, V, K, PF, FLIP, M>
    "fwd:nhwc_rowwalk_k3s1": [r"k_nhwc_s1<[\w ]+, \d+, 3, \d+, false, 1>"],
    "bwd_data:nhwc_rowwalk_k3s1_flip": [r"k_nhwc_s1<[\w ]+, \d+, 3, \d+, true, 1>"],
    "fwd:nhwc_rowwalk_k5s1": [r"k_nhwc_s1<[\w ]+, \d+, 5, \d+, false, 1>", r"k_nhwc_s1_2col<[\w ]+, \d+, 5, \d+, false,"],
    "bwd_data:nhwc_rowwalk_k5s1_flip": [r"k_nhwc_s1<[\w ]+, \d+, 5, \d+, true, 1>", r"k_nhwc_s1_2col<[\w ]+, \d+, 5, \d+, true,"],
    "fwd:nhwc_rowwalk_k3s1_m2": [r"k_nhwc_s1<[\w ]+, \d+, 3, \d+, false, 2>"],
    "bwd_data:nhwc_rowwalk_k3s1_flip_m2": [r"k_nhwc_s1<[\w ]+, \d+, 3, \d+, true, 2>"],
    "fwd:nhwc_rowwalk_fwd_k3s2": [r"k_nhwc_fwd_k3s2<"],
    "bwd_data:nhwc_rowwalk_bwd_data_k3s2": [r"k_nhwc_bwd_data_k3s2<"],
    # k_nhwc_bwd_filter<T, V, K, S, PF, M, FLAT>
    "bwd_filter:nhwc_bwd_filter_k3s1": [r"k_nhwc_bwd_filter<[\w ]+, \d+, 3, 1, \d+, 1, \w+>", r"k_nhwc_bwd_filter_dot2<\d+, 3>"],
    "bwd_filter:nhwc_bwd_filter_k3s2": [r"k_nhwc_bwd_filter<[\w ]+, \d+, 3, 2, \d+, 1, \w+>"],
    "bwd_filter:nhwc_bwd_filter_k5s1": [r"k_nhwc_bwd_filter<[\w ]+, \d+, 5, 1, \d+, 1, \w+>", r"k_nhwc_bwd_filter_dot2<\d+, 5>"],
    "bwd_filter:nhwc_bwd_filter_k3s1_m2": [r"k_nhwc_bwd_filter<[\w ]+, \d+, 3, 1, \d+, 2, \w+>"],
    # k_nchwd_s1<T, V, K, PF, FLIP, RS> (RS > 0: whole-line write-out)
    # bf16: k_nchwd_s1_bf16x8<V, K, PF, FLIP, RS> (packed pairs)
    "fwd:nchw_rowwalk_k3s1": [r"k_nchwd_s1<[\w ]+, \d+, 3, \d+, false[,>]", r"k_nchwd_s1_bf16x8<\d+, 3, \d+, false,"],
    "bwd_data:nchw_rowwalk_k3s1_flip": [r"k_nchwd_s1<[\w ]+, \d+, 3, \d+, true[,>]", r"k_nchwd_s1_bf16x8<\d+, 3, \d+, true,"],
    "fwd:nchw_rowwalk_k5s1": [r"k_nchwd_s1<[\w ]+, \d+, 5, \d+, false[,>]", r"k_nchwd_s1_bf16x8<\d+, 5, \d+, false,"],
    "bwd_data:nchw_rowwalk_k5s1_flip": [r"k_nchwd_s1<[\w ]+, \d+, 5, \d+, true[,>]", r"k_nchwd_s1_bf16x8<\d+, 5, \d+, true,"],
    "fwd:nchw_rowwalk_fwd_k3s2": [r"k_nchwd_fwd_k3s2<"],
    "bwd_data:nchw_rowwalk_bwd_data_k3s2": [r"k_nchwd_bwd_data_k3s2<"],
    "bwd_filter:nchw_rowwalk_bwd_filter_k3s1": [r"k_nchwd_bwd_filter_k3<[\w ]+, \d+, 1>", r"k_nchwd_bwd_filter_s1_bf16<\d+, 3>"],
    "bwd_filter:nchw_rowwalk_bwd_filter_k3s2": [r"k_nchwd_bwd_filter_k3<[\w ]+, \d+, 2>"],
    "bwd_filter:nchw_rowwalk_bwd_filter_k5s1": [r"k_nchwd_bwd_filter_s1<[\w ]+, \d+, 5>", r"k_nchwd_bwd_filter_s1_bf16<\d+, 5>"],
    # k_nchws_fwd<T, K, S, W, FLIP, INPLACE, CG>, k_nchws_bwd_filter<T, K, S, W, CG> (CG = 1: depthwise)
    "fwd:nchw_smallplane_k3s1": [r"k_nchws_fwd<[\w ]+, 3, 1, \d+, false, \w+, 1>"],
    "bwd_data:nchw_smallplane_k3s1_flip": [r"k_nchws_fwd<[\w ]+, 3, 1, \d+, true, \w+, 1>"],
    "fwd:nchw_smallplane_fwd_k3s2": [r"k_nchws_fwd<[\w ]+, 3, 2, \d+, false, \w+, 1>"],
    "bwd_data:nchw_smallplane_bwd_data_k3s2": [r"k_nchws_bwd_data_s2<"],
    "bwd_filter:nchw_smallplane_bwd_filter_k3s1": [r"k_nchws_bwd_filter<[\w ]+, 3, 1, \d+, 1>"],
    "bwd_filter:nchw_smallplane_bwd_filter_k3s2": [r"k_nchws_bwd_filter<[\w ]+, 3, 2, \d+, 1>"],
    "fwd:nchw_smallplane_k5s1": [r"k_nchws_fwd<[\w ]+, 5, 1, \d+, false, \w+, 1>"],
    "bwd_data:nchw_smallplane_k5s1_flip": [r"k_nchws_fwd<[\w ]+, 5, 1, \d+, true, \w+, 1>"],
    "bwd_filter:nchw_smallplane_bwd_filter_k5s1": [r"k_nchws_bwd_filter<[\w ]+, 5, 1, \d+, 1>"],
    # whole backward pass in one kernel (dwconv_bwd)
    # k_nhwc_bwd_fused_k3s1<T, V, PF, M>
    "bwd:nhwc_bwd_fused_k3s1": [r"k_nhwc_bwd_fused_k3s1<[\w ]+, \d+, \d+, 1>"],
    "bwd:nhwc_bwd_fused_k3s1_m2": [r"k_nhwc_bwd_fused_k3s1<[\w ]+, \d+, \d+, 2>"],
    "bwd:nhwc_bwd_fused_k3s2": [r"k_nhwc_bwd_fused_k3s2<"],
    "bwd:nchw_bwd_fused_k3s1": [r"k_nchwd_bwd_fused_k3s1<"],
    "bwd:nchw_bwd_fused_k3s2": [r"k_nchwd_bwd_fused_k3s2<"],
    "bwd:nchw_smallplane_bwd_fused_k3s1": [r"k_nchws_bwd_fused<"],
    "bwd:nchw_smallplane_bwd_fused_k3s2": [r"k_nchws_bwd_fused_s2<"],
    # group convolution: k_gconv_nchw_s1<T, V, OB, R, FLIP, SHFL>, k_gconv_nhwc_s1<T, CG, OB, GPL, PF, FLIP>
    "fwd:group_nchw_rowwalk_k3s1": [r"k_gconv_nchw_s1<[\w ]+, \d+, \d+, \d+, false[,>]"],
    "bwd_data:group_nchw_rowwalk_k3s1_flip": [r"k_gconv_nchw_s1<[\w ]+, \d+, \d+, \d+, true[,>]"],
    "bwd_filter:group_nchw_bwd_filter_k3s1": [r"k_gconv_nchw_bwd_filter<"],
    "fwd:group_nchw_smallplane_k3s1": [r"k_nchws_fwd<[\w ]+, 3, 1, \d+, false, \w+, [248]>"],
    "bwd_data:group_nchw_smallplane_k3s1_flip": [r"k_nchws_fwd<[\w ]+, 3, 1, \d+, true, \w+, [248]>"],
    "fwd:group_nchw_smallplane_mfma_k3s1": [r"k_gconv_nchws_mfma_fwd<[\w ]+, \d+, \d+, \d+, false>"],
    "bwd_data:group_nchw_smallplane_mfma_k3s1_flip": [r"k_gconv_nchws_mfma_fwd<[\w ]+, \d+, \d+, \d+, true>"],
    "bwd_filter:group_nchw_smallplane_mfma_bwd_filter_k3s1": [r"k_gconv_nchws_mfma_bwd_filter<[\w ]+, \d+, \d+, \d+, false>"],
    "bwd_filter:group_nhwc_mfma_bwd_filter_k3s1": [r"k_gconv_nhwc_tr_bwd_filter<"],
    "bwd_filter:group_nhwc_lds_mfma_bwd_filter_k3s1": [r"k_gconv_nchws_mfma_bwd_filter<[\w ]+, \d+, \d+, \d+, true>"],
    "bwd_filter:group_nchw_smallplane_bwd_filter_k3s1": [r"k_nchws_bwd_filter<[\w ]+, 3, 1, \d+, [248]>"],
    # k_gconv_nhwc_xchg<T, CG, V, PF, FLIP>: the lane-exchange walk (groups of 4 or 8 channels)
    "fwd:group_nhwc_rowwalk_k3s1": [r"k_gconv_nhwc_s1<[\w ]+, \d+, \d+, \d+, \d+, false>", r"k_gconv_nhwc_xchg<[\w ]+, \d+, \d+, \d+, false>"],
    "bwd_data:group_nhwc_rowwalk_k3s1_flip": [r"k_gconv_nhwc_s1<[\w ]+, \d+, \d+, \d+, \d+, true>", r"k_gconv_nhwc_xchg<[\w ]+, \d+, \d+, \d+, true>"],
    # k_gconv_nhwc_mfma<T, CG, FLIP, PF>
    "fwd:group_nhwc_mfma_k3s1": [r"k_gconv_nhwc_mfma<[\w ]+, \d+, false, \d+>"],
    "bwd_data:group_nhwc_mfma_k3s1_flip": [r"k_gconv_nhwc_mfma<[\w ]+, \d+, true, \d+>"],
    "bwd_filter:group_nhwc_bwd_filter_k3s1": [r"k_gconv_nhwc_bwd_filter<", r"k_gconv_nhwc_bwd_filter_dot2<", r"k_gconv_nhwc_xchg_bwd_filter<"],
}


def _one(pattern):
    files = glob.glob(pattern)
    if not files:
        sys.exit("no file matches " + pattern)
    return files[0]


def short(name):
    name = re.sub(r"\(.*$", "", name)
    return name.replace("void dwc::", "").replace("dwc::", "")


def _workload_keys(config, fused=False):
    """bench.py's "<pass>:<variant>" keys of a workload: launches per step and algorithmic bytes per step of each.
    fused: the step of `bench.py --fused-bwd`, whose backward pass is one dwconv_bwd call per layer (key "bwd:<variant>",
    2|x| + |y| elements) where a fused kernel exists and the two separate passes elsewhere."""
    import paper_1803_09926_amd as dw
    from paper_1803_09926_amd import workloads as wl
    cfg = wl.config(config)
    esz = 4 if cfg["dtype"] == wl.F32 else 2
    launches, nbytes = {}, {}
    for layout in cfg["layouts"]:
        for layer, repeat in cfg["layers"]:
            if layer.cg > 1:
                d = dw.group_desc(cfg["N"], layer.C, layer.H, layer.W, layer.K, layer.stride, layer.pad, layer.groups,
                                  layer.O, layout, cfg["dtype"])
                vname = dw.gconv_variant_name
            else:
                d = dw.desc(cfg["N"], layer.C, layer.H, layer.W, layer.K, layer.stride, layer.pad, layer.mult, layout, cfg["dtype"])
                vname = dw.variant_name
            whole = vname(d, 3) if (fused and layer.cg == 1) else "separate"
            for which, pname in enumerate(("fwd", "bwd_data", "bwd_filter")):
                if which > 0 and whole != "separate":
                    continue
                key = pname + ":" + vname(d, which)
                launches[key] = launches.get(key, 0) + repeat
                nbytes[key] = nbytes.get(key, 0) + repeat * layer.pass_bytes(cfg["N"], esz)
            if whole != "separate":
                key = "bwd:" + whole
                launches[key] = launches.get(key, 0) + repeat
                nbytes[key] = nbytes.get(key, 0) + repeat * (2 * layer.x_elems(cfg["N"]) + layer.y_elems(cfg["N"])) * esz
    return launches, nbytes


def stats(d, config=None, fused=False):
    rows = list(csv.DictReader(open(_one(os.path.join(d, "*kernel_stats.csv")))))
    rows = [r for r in rows if "dwc::" in r["Name"]]
    total = sum(int(r["TotalDurationNs"]) for r in rows)
    print("%-64s %7s %12s %12s %10s %10s %6s" % ("kernel", "calls", "total_us", "avg_us", "min_us", "max_us", "%"))
    for r in sorted(rows, key=lambda r: -int(r["TotalDurationNs"])):
        print("%-64s %7d %12.1f %12.2f %10.2f %10.2f %6.2f" % (
            short(r["Name"])[:64], int(r["Calls"]), int(r["TotalDurationNs"]) / 1e3, float(r["AverageNs"]) / 1e3,
            int(r["MinNs"]) / 1e3, int(r["MaxNs"]) / 1e3, 100.0 * int(r["TotalDurationNs"]) / total))
    print("sum over the library's kernels: %.1f us" % (total / 1e3))
    # bench.py's keys: launches and average duration inside the profiled steps of the kernel(s) behind each key
    print("# bench.py keys: instep <pass:variant> <dispatches> <average us per dispatch, inside the profiled steps>")
    per_key = {}
    for key, pats in VARIANT_KERNELS.items():
        ks = [r for r in rows if any(re.search(p, short(r["Name"])) for p in pats)]
        if not ks:
            continue
        calls = sum(int(r["Calls"]) for r in ks)
        tot = sum(int(r["TotalDurationNs"]) for r in ks) / 1e3
        per_key[key] = (calls, tot)
        print("instep %s %d %.2f" % (key, calls, tot / calls))
    if config is None:
        return
    # per layout and pass: time per step from the trace against the algorithmic bytes of the workload
    from paper_1803_09926_amd import workloads as wl
    cfg = wl.config(config)
    launches, nbytes = _workload_keys(config, fused)
    missing = [k for k in launches if k not in per_key]
    if missing:
        print("# keys of the workload with no kernel in the trace: " + ", ".join(missing))
    known = [k for k in launches if k in per_key]
    steps = sorted(per_key[k][0] / launches[k] for k in known)[len(known) // 2]
    red = [r for r in rows if "k_reduce_partials" in r["Name"]]
    red_us = sum(int(r["TotalDurationNs"]) for r in red) / 1e3
    nfilter = sum(v for k, v in launches.items() if k.startswith("bwd_filter:") or k.startswith("bwd:"))
    print("# workload %s: %.0f steps in the trace; per layout and pass, per step: kernel time, algorithmic bytes, rate" % (cfg["name"], steps))
    print("# (bwd_filter, and bwd = the whole backward pass in one call: stage 1 + its share of the stage-2 launches k_reduce_partials, split by launch count)")
    print("%-6s %-11s %10s %12s %9s %7s" % ("layout", "pass", "us/step", "MB/step", "GB/s", "%peak"))
    grand_us = grand_b = 0.0
    for lay in ("nchw", "nhwc"):
        for pname in ("fwd", "bwd_data", "bwd_filter", "bwd"):
            ks = [k for k in known if k.startswith(pname + ":") and ("_" + lay + "_" in "_" + k.split(":")[1] + "_")]
            if not ks:
                continue
            us = sum(per_key[k][1] for k in ks) / steps
            if pname in ("bwd_filter", "bwd") and nfilter:
                us += red_us / steps * sum(launches[k] for k in ks) / nfilter
            b = sum(nbytes[k] for k in ks)
            grand_us += us; grand_b += b
            print("pass %-6s %-11s %10.1f %12.1f %9.1f %7.2f" % (lay, pname, us, b / 1e6, b / us / 1e3, b / us / 1e3 / 80.0))
    if grand_us:
        print("pass %-6s %-11s %10.1f %12.1f %9.1f %7.2f" % ("all", "all", grand_us, grand_b / 1e6, grand_b / grand_us / 1e3, grand_b / grand_us / 1e3 / 80.0))


def _counter(d, cname):
    rows = [r for r in csv.DictReader(open(_one(os.path.join(d, "*counter_collection.csv")))) if r["Counter_Name"] == cname]
    cal = [float(r["Counter_Value"]) for r in rows if "copyBuffer" in r["Kernel_Name"]]
    if not cal:
        sys.exit("no calibration copy in " + d + " (run bench.py with --calibrate-copy)")
    unit = float(1 << 30) / (sum(cal) / len(cal))
    per = {}
    for r in rows:
        if "dwc::" not in r["Kernel_Name"]:
            continue
        per.setdefault(short(r["Kernel_Name"]), []).append(float(r["Counter_Value"]) * unit)
    return unit, cal, per


def traffic(dfetch, dwrite, config=None):
    fu, fcal, fper = _counter(dfetch, "FETCH_SIZE")
    wu, wcal, wper = _counter(dwrite, "WRITE_SIZE")
    print("# calibration: a device copy of 2^30 bytes reads FETCH_SIZE = %s and writes WRITE_SIZE = %s" % (fcal, wcal))
    print("# scale: %.1f bytes per FETCH_SIZE unit, %.1f bytes per WRITE_SIZE unit" % (fu, wu))
    print("# per kernel: mean HBM bytes per dispatch (fetch, write, sum) over all its dispatches")
    print("%-64s %7s %14s %14s %14s" % ("kernel", "calls", "fetch_B", "write_B", "total_B"))
    for k in sorted(fper):
        f = sum(fper[k]) / len(fper[k]); w = sum(wper.get(k, [0.0])) / max(1, len(wper.get(k, [])))
        print("%-64s %7d %14.0f %14.0f %14.0f" % (k[:64], len(fper[k]), f, w, f + w))
    print("# bench.py keys: mean HBM bytes per launch over every dispatch of the kernel(s) behind the key")
    print("# (for bwd_filter: stage 1 only; the stage-2 kernel k_reduce_partials is listed above)")
    measured = {}
    for key, pats in VARIANT_KERNELS.items():
        ks = [k for k in fper if any(re.search(p, k) for p in pats)]
        if not ks:
            continue
        calls = sum(len(fper[k]) for k in ks)
        val = (sum(sum(fper[k]) for k in ks) + sum(sum(wper.get(k, [])) for k in ks)) / calls
        print("traffic %s %.0f" % (key, val))
        measured[key] = val
    if config is None:
        return
    # measured HBM bytes per launch against the algorithmic bytes of the same launches (mean over the key's layers)
    launches, nbytes = _workload_keys(config)
    print("# measured HBM traffic over algorithmic bytes (|x| + |y|) per launch, per bench.py key of workload %d" % config)
    print("%-48s %14s %14s %7s" % ("key", "measured_B", "algorithmic_B", "ratio"))
    for key in measured:
        if key in launches:
            alg = nbytes[key] / launches[key]
            print("ratio %-42s %14.0f %14.0f %7.3f" % (key, measured[key], alg, measured[key] / alg))


def pmc(d, pattern=""):
    """Mean value per dispatch of every counter of a `rocprofv3 --pmc` run, per kernel of the library whose name contains
    `pattern`; with SQ_VALU_MFMA_BUSY_CYCLES and GRBM_GUI_ACTIVE in the run also the share of time the matrix cores are
    busy (busy cycles summed over the 1024 SIMDs against the active cycles summed over the 8 XCDs)."""
    files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        sys.exit("no *counter_collection.csv under %s" % d)
    per = {}
    for r in csv.DictReader(open(files[0])):
        n = r["Kernel_Name"]
        if "dwc::" not in n or pattern not in n:
            continue
        n = re.sub(r"\(.*$", "", n).replace("void dwc::", "")
        per.setdefault(n, {}).setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
    ctrs = sorted({c for v in per.values() for c in v})
    print("# mean per dispatch; counters: " + " ".join(ctrs))
    print("%-58s %5s " % ("kernel", "n") + " ".join("%18s" % c[-18:] for c in ctrs) + "  mfma_busy")
    for k in sorted(per):
        v = per[k]
        mean = {c: sum(v[c]) / len(v[c]) for c in v}
        busy = ""
        if "SQ_VALU_MFMA_BUSY_CYCLES" in mean and mean.get("GRBM_GUI_ACTIVE"):
            busy = "%8.1f %%" % (100.0 * mean["SQ_VALU_MFMA_BUSY_CYCLES"] / (mean["GRBM_GUI_ACTIVE"] / 8.0 * 1024.0))
        print("%-58s %5d " % (k[:58], len(v[ctrs[0]])) + " ".join("%18.0f" % mean.get(c, 0.0) for c in ctrs) + "  " + busy)


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(sys.argv[2], int(sys.argv[3]) if len(sys.argv) >= 4 else None, fused=len(sys.argv) >= 5 and sys.argv[4] == "fused")
    elif len(sys.argv) >= 3 and sys.argv[1] == "pmc":
        pmc(sys.argv[2], sys.argv[3] if len(sys.argv) >= 4 else "")
    elif len(sys.argv) >= 4 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], int(sys.argv[4]) if len(sys.argv) >= 5 else None)
    else:
        sys.exit(__doc__)
