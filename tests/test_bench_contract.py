"""The benchmark's command-line contract: one GPU only, one JSON line with the agreed keys."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KEYS = {"metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
        "scaling", "vs_baseline", "dtype", "data", "config", "roofline"}


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    assert p.returncode == 2 and "ONE GPU" in p.stderr and p.stdout.strip() == ""


def test_build_entry_point_compiles_and_imports():
    """__graft_entry__.build() as a fresh process runs it: compiles the library for gfx950,
    the oracle and the native driver, imports the package and checks the ABI it loaded."""
    p = subprocess.run([sys.executable, "-c", "import __graft_entry__ as g; g.build(); print('built')"],
                       cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=600)
    assert p.returncode == 0 and p.stdout.strip().endswith("built"), p.stderr[-2000:]


def test_measured_traffic_matches_the_algorithmic_bytes_or_is_absent():
    sys.path.insert(0, ROOT)
    import bench
    from synth import WORKLOADS
    w = WORKLOADS["70b_zero3"]
    t = bench.measured_traffic(w, 1 << 28)
    assert t is None or abs(t / (42.0 * (1 << 28)) - 1.0) < 0.01
    assert bench.measured_traffic(WORKLOADS["tiny"], 1 << 18) is None     # no counters for this workload
    assert bench.bytes_per_elem(w) == 42 and bench.bytes_per_elem(WORKLOADS["13b_clip"], True) == 58
    assert bench.bytes_per_elem(WORKLOADS["tiny"]) == 34
    assert bench.bytes_per_elem(WORKLOADS["7b_zero1"]) == 28
    # three accumulation passes (20, 24, 24) and the update from the last micro-batch and the
    # accumulator (16 + 4 + 12 read, 14 written)
    assert bench.bytes_per_elem(WORKLOADS["7b_accum4"]) == 20 + 24 + 24 + 46 == 114


@pytest.mark.gpu
@pytest.mark.parametrize("workload", ["tiny", "gpt2s"])
def test_json_line(workload):
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", workload,
                        "--steps", "3", "--warmup", "1", "--cpu-baseline-seconds", "2"],
                       stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, text=True, timeout=280)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert KEYS <= set(d) and "cpu_baseline" in d
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["vs_baseline"] is None
    assert d["unit"] == "elements/s" and d["dtype"] == "f32" and d["data"] == "synthetic"
    assert d["config"]["workload"] == workload and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12 and r["achieved"] > 0
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["sample"]
    assert d["value"] > c["value"]


@pytest.mark.gpu
@pytest.mark.parametrize("workload", ["13b_clip", "7b_zero2_f16", "7b_zero1", "7b_accum4", "7b_verify"])
def test_json_line_of_the_other_workloads(workload):
    """The other bench.py workloads still run and print one well-formed line (no CPU leg:
    these shards are large and the oracle baseline is covered above)."""
    import torch
    if torch.cuda.mem_get_info()[0] < 120e9:
        pytest.skip("needs a device with 120 GB free")
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", workload,
                        "--steps", "2", "--warmup", "1", "--no-cpu-baseline"],
                       stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=280)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert KEYS <= set(d) and d["config"]["workload"] == workload and d["value"] > 0
    r = d["roofline"]
    assert r["peak"] == 8000.0 and 0.5 < r["frac"] < 1.0     # an HBM-bound kernel on this part


@pytest.mark.gpu
@pytest.mark.parametrize("layout", ["packed", "flat"])
def test_json_line_of_the_offloaded_workload(layout):
    """The offloaded workload is bound by the host link: its line carries that roofline and
    the probe of plain pinned copies it is measured against."""
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "7b_offload",
                        "--offload-layout", layout, "--steps", "2", "--warmup", "1", "--no-cpu-baseline"],
                       stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=280)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert KEYS <= set(d) and d["config"]["workload"] == "7b_offload" and d["value"] > 0
    assert d["config"]["host_layout"] == layout
    r = d["roofline"]
    assert r["bound"].startswith("host link") and r["peak"] == 64.0 and 0.0 < r["frac"] < 1.0
    assert d["extras"]["link_probe"]["both_directions_ms"] > 0

