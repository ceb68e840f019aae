"""Host-side checks of bench.py's contract that need no GPU: the metric is the one the benchmark spec names, the
workload tables carry the sizes the metric is computed from, and a run on more than one GPU is refused."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_metric_and_workload_are_the_ones_the_baseline_names():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2104_10949_amd import workloads as wl
    base = json.load(open(os.path.join(ROOT, "BASELINE.json")))
    assert bench.METRIC == base["metric"]
    assert bench.INT8_PEAK_TOPS == 5000.0
    # the timed configuration is the one with the most ring MACs among the five
    macs = {c: sum(L.gemm[0] * L.gemm[1] * L.gemm[2] * L.repeat for L in wl.config_layers(c)) for c in (1, 2, 3, 4, 5)}
    assert max(macs, key=macs.get) == bench.WORKLOAD_CONFIG
    # 72 signed-byte digit MACs per (m, n, k): two ring products of 36 digit pairs each (l + m <= 7)
    assert bench.DIGIT_MACS_PER_RING_MAC_TRIPLE == 2 * sum(1 for l in range(8) for m in range(8) if l + m <= 7)


def test_layer_tables_match_the_configurations():
    sys.path.insert(0, ROOT)
    from paper_2104_10949_amd import workloads as wl
    assert [L.gemm for L in wl.config_layers(1)] == [(256, 256, 256)]
    assert [L.gemm for L in wl.config_layers(2)] == [(128, 128, 784), (128, 128, 128), (128, 10, 128)]
    c4 = wl.config_layers(4)
    assert len(c4) == 16 and sum(L.kind == "conv" for L in c4) == 13
    assert c4[1].gemm == (131072, 64, 576) and c4[-3].gemm == (32, 512, 8192) and c4[-1].gemm == (32, 200, 512)
    c5 = wl.config_layers(5)
    assert sum(L.repeat for L in c5 if L.kind == "conv") == 53   # layers of one shape are listed once, with a count
    assert c5[0].gemm == (100352, 64, 147) and c5[-1].gemm == (8, 1000, 2048)


def test_more_than_one_gpu_is_refused_before_anything_touches_a_device():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2
    assert r.stdout.strip() == ""
    assert "ONE GPU" in r.stderr


def test_traffic_constants_are_the_ones_the_committed_counter_summary_holds():
    """bench.py quotes the HBM bytes per launch from the rocprofv3 counter summary: both must say the same."""
    import re
    sys.path.insert(0, ROOT)
    import bench
    t = bench.PROFILED_TRAFFIC_CONFIG4
    text = open(os.path.join(ROOT, t["source"])).read()
    m = re.search(r"scaled bytes per dispatch:\s*([\d.]+) MB read,\s*([\d.]+) MB written", text)
    assert m, "summary line of the product kernels not found"
    assert abs(float(m.group(1)) * 1e6 - t["read_bytes_per_launch"]) < 0.05e6
    assert abs(float(m.group(2)) * 1e6 - t["write_bytes_per_launch"]) < 0.05e6
    m = re.search(r"([\d.]+) MB per dispatch", text)
    assert m and abs(float(m.group(1)) * 1e6 - t["algorithmic_bytes_per_launch"]) < 0.05e6
    # the conversion pass: the to_planes_kernel line holds FETCH_SIZE and WRITE_SIZE in KiB per dispatch (x 2.000, x 1.000)
    m = re.search(r"to_planes_kernel\S*\s+\d+\s+([\d.]+)\s+([\d.]+)", text)
    conv = t["conversion_pass_per_scratch_route_layer"]
    assert m and abs(float(m.group(1)) * 1024 * 2.0 - conv["read_bytes"]) < 0.05e6
    assert abs(float(m.group(2)) * 1024 * 1.0 - conv["write_bytes"]) < 0.05e6
