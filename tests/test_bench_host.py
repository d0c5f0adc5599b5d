"""Host-side checks of the measurement code: bench.py's argument contract, the profile-summary tool on a small
synthetic rocprofv3 table, and that the committed summaries carry what the bench line reads from them."""
import csv
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_workload_keys_cover_the_headline_bytes():
    from paper_1803_09926_amd import rocprof_summary as rs
    launches, nbytes = rs._workload_keys(2)
    assert sum(launches.values()) == 13 * 3 * 2                      # 13 layers, three passes, two layouts
    assert sum(nbytes.values()) == 15336996864                       # 2 layouts x 3 passes x 2.556 GB
    assert all(":" in k and not k.endswith(":generic") for k in launches)


def test_stats_summary_on_a_synthetic_trace(tmp_path, capsys):
    from paper_1803_09926_amd import rocprof_summary as rs
    rows = [
        ("void dwc::k_nhwc_s1<float, 4, 3, 4, false, 1>(dwc::Geom, float const*)", 18, 720000),
        ("void dwc::k_nhwc_bwd_filter<float, 4, 3, 1, 2, 1, false>(dwc::Geom, float const*)", 18, 540000),
        ("void dwc::k_reduce_partials<8>(float const*, int, int, float*)", 26, 117000),
        ("some_other_kernel(int)", 5, 1000),
    ]
    with open(tmp_path / "b_kernel_stats.csv", "w", newline="") as f:
        wr = csv.writer(f)
        wr.writerow(["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"])
        for name, calls, tot in rows:
            wr.writerow([name, calls, tot, tot / calls, 0.0, 1000, 90000, 0.0])
    rs.stats(str(tmp_path))
    out = capsys.readouterr().out
    assert "some_other_kernel" not in out                             # only the library's kernels
    assert "instep fwd:nhwc_rowwalk_k3s1 18 40.00" in out             # 720 us over 18 dispatches
    assert "instep bwd_filter:nhwc_bwd_filter_k3s1 18 30.00" in out


def test_committed_summaries_feed_the_bench_line():
    bench = _bench_module()
    prof = bench.stored_profile("mobilenet_v1_dw_b128_f32_nchw_nhwc", "fwd:nhwc_rowwalk_k3s1")
    assert prof["traffic"] and 1.0 <= prof["traffic"] / 176976327 < 1.1      # measured HBM bytes per launch, close to algorithmic
    assert prof["in_step_avg_us"] and 20.0 < prof["in_step_avg_us"] < 60.0
    assert prof["traffic_file"].startswith("profiles/hbm_traffic_") and prof["stats_file"].startswith("profiles/kernel_stats_")
    for wl_name in ("mobilenet_v1_dw_b64_f32_nhwc", "xception_dw_b32_f32_nhwc", "mobilenet_v1_dw_b256_bf16"):
        p = bench.stored_profile(wl_name, "fwd:nhwc_rowwalk_k3s1")
        assert p["traffic"] and p["in_step_avg_us"], wl_name


def test_profiles_hold_only_short_text_summaries():
    for name in os.listdir(os.path.join(ROOT, "profiles")):
        path = os.path.join(ROOT, "profiles", name)
        assert name.endswith((".txt", ".md")), name
        assert os.path.getsize(path) < 32 * 1024, name
        head = open(path).read(4000)
        assert "rocprofv3" in head or "python3 -m" in head, name      # the command that made it
