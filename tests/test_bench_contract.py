"""bench.py's output contract, checked on the smallest workloads (GPU), its refusal of several GPUs (anywhere), and the
stand-alone C program that uses the library without Python."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_traffic_record_is_tied_to_sources_and_plan(tmp_path, monkeypatch):
    """roofline.traffic is reported only from a counter record taken on the present library sources and the same plan."""
    sys.path.insert(0, ROOT)
    import bench
    rec = {"workloads": {"w": {"fetch_size_kib": 1000.0, "write_size_kib": 2000.0, "fetch_scale": 2.0, "write_scale": 1.0,
                               "n_tiles": 7, "algorithmic_bytes": 4096000, "source_hash": bench.source_hash(), "profile": "profiles/x.md"}}}
    f = tmp_path / "t.json"
    f.write_text(json.dumps(rec))
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(f))
    good = {"n_tiles": 7, "bytes_read": 2048000, "bytes_written": 2048000}
    assert bench.measured_traffic("w", good) == (4096000, "profiles/x.md")
    assert bench.measured_traffic("w", dict(good, n_tiles=8))[0] is None
    assert bench.measured_traffic("other", good)[0] is None
    rec["workloads"]["w"]["source_hash"] = "0" * 16
    f.write_text(json.dumps(rec))
    assert bench.measured_traffic("w", good)[0] is None
    # the committed record is well-formed (whether it still matches the sources is bench.py's business at run time)
    with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as fh:
        committed = json.load(fh)["workloads"]
    assert all({"fetch_size_kib", "write_size_kib", "fetch_scale", "write_scale", "n_tiles", "algorithmic_bytes", "source_hash",
                "profile"} <= set(v) for v in committed.values()) and "gpt6.7b_(8,1,1)->(1,8,1)" in committed


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode != 0 and "one GPU" in r.stderr and not r.stdout.strip()


@pytest.mark.gpu
@pytest.mark.parametrize("workload", ["tiny_2L_h256_(2,1,1)->(4,2,1)", "dataset_1e8_D6->D4"])
def test_bench_prints_one_json_line_with_the_contract_fields(cuda, workload):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", workload, "--steps", "3", "--warmup", "1"],
                       capture_output=True, text=True, cwd=ROOT, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["metric"] == "reshard_GBps_state_bytes_read_plus_written" and d["unit"] == "GB/s"
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["scaling"] == "weak" and d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] in ("u8", "u64")
    assert d["config"]["workload"] == workload and "model" not in d["config"]
    assert d["value"] > 0 and d["ms_per_step"] > 0
    assert abs(d["value"] - (d["config"]["state_bytes_read"] + d["config"]["state_bytes_written"]) / d["ms_per_step"] / 1e6) <= 0.01 * d["value"] + 0.1
    roof = d["roofline"]
    assert roof["bound"] == "hbm" and roof["unit"] == "GB/s" and roof["peak"] == 8000.0 and "traffic" in roof
    # traffic comes from the counter record under profiles/ and only while that record matches the sources and the plan
    if roof["traffic"] is None:
        assert isinstance(roof["traffic_from"], str) and roof["traffic_from"]
    else:
        assert roof["traffic_from"].startswith("profiles/") and os.path.exists(os.path.join(ROOT, roof["traffic_from"]))
        assert 0.99 < roof["traffic"] / roof["algorithmic_bytes_per_launch"] < 1.05
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["unit"] == "GB/s" and cpu["value"] > 0 and cpu["cores"] >= 1 and cpu["sample"]
    assert cpu["gpu_matches_oracle_on_sample"] is True


@pytest.mark.gpu
def test_bench_in_process_comparison_mode(cuda):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "tiny_2L_h256_(2,1,1)->(4,2,1)", "--ab",
                        ";streams=1,chunk=1;tile_bytes=4096,occupancy=2"], capture_output=True, text=True, cwd=ROOT, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads([l for l in r.stdout.splitlines() if l.strip()][-1])
    assert [x["setting"] for x in d["settings"]] == ["default", "streams=1,chunk=1", "tile_bytes=4096,occupancy=2"]
    assert all(len(x["rounds"]) == 3 and x["best"] > 0 for x in d["settings"])
    assert d["settings"][2]["n_tiles"] > d["settings"][0]["n_tiles"]
    bad = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--ab", "nonsense=1"], capture_output=True, text=True, cwd=ROOT)
    assert bad.returncode != 0 and "unknown key" in bad.stderr


@pytest.mark.gpu
def test_c_abi_without_python_or_torch(cuda):
    """paper_2312_05181_amd/examples/reshard_selftest.cpp, built next to the library: plans, executes and checks a reshard through the
    C ABI alone, with the system's HIP runtime."""
    exe = os.path.join(ROOT, "paper_2312_05181_amd", "tpx_selftest")
    assert os.path.exists(exe), "build it with python -m paper_2312_05181_amd.build"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-2000:]
    assert " 0 wrong" in r.stdout
