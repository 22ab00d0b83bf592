"""bench.py's output contract: one JSON line on stdout with the agreed keys, and a refusal of more than one GPU."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_tiny_run_prints_one_json_line_with_the_agreed_keys():
    print("bench.py --tiny --steps 2 --warmup 1", flush=True)
    r = subprocess.run([sys.executable, BENCH, "--tiny", "--steps", "2", "--warmup", "1"], capture_output=True, text=True,
                       timeout=110, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, r.stdout
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 2 and out["warmup"] == 1
    assert out["unit"] == "GB/s" and out["higher_is_better"] is True and out["vs_baseline"] is None
    assert out["dtype"] == "u16" and out["data"] == "synthetic" and "workload" in out["config"]
    assert out["value"] > 0 and out["ms_per_step"] > 0
    roof = out["roofline"]
    assert roof["bound"] == "hbm" and roof["unit"] == "GB/s" and roof["peak"] == 8000.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3 and "traffic" in roof
    cpu = out["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] == 1 and cpu["value"] > 0 and cpu["unit"] == "GB/s" and cpu["sample"]
    assert out["checked"] is True
    ra = out["roofline_apply"]
    assert ra["bound"] == "hbm" and ra["kernel"] == "apply_kernel" and abs(ra["frac"] - ra["achieved"] / ra["peak"]) < 1e-3
    assert "traffic" in ra and ra["line_model_gbs"] > 0
    for key in ("cpu_baseline_all_cores", "other_configs", "rotating_snapshot"):
        assert key in out, key


def test_traffic_figures_follow_the_kernel_sources(tmp_path, monkeypatch):
    """The HBM-traffic figures of the JSON line come from a tracked counter summary and are withheld as soon as
    the kernel sources differ from the ones the summary was measured with."""
    sys.path.insert(0, ROOT)
    import bench
    good = tmp_path / "traffic.txt"
    good.write_text("# comment\nworkload = w\nsources_sha256 = %s\nextract_read_bytes = 10\nextract_written_bytes = 3\n"
                    "apply_read_bytes = 2\napply_written_bytes = 9\n" % bench.kernel_source_hash())
    monkeypatch.setattr(bench, "TRAFFIC_SUMMARY", str(good))
    assert bench.measured_traffic("w") == {"extract": (10.0, 3.0), "apply": (2.0, 9.0)}
    assert bench.measured_traffic("another workload") is None
    stale = tmp_path / "stale.txt"
    stale.write_text(good.read_text().replace(bench.kernel_source_hash(), "0" * 64))
    monkeypatch.setattr(bench, "TRAFFIC_SUMMARY", str(stale))
    assert bench.measured_traffic("w") is None
    monkeypatch.setattr(bench, "TRAFFIC_SUMMARY", str(tmp_path / "missing.txt"))
    assert bench.measured_traffic("w") is None


def test_all_cores_oracle_leg_runs_disjoint_bucket_runs_on_host_threads():
    """bench.py's all-cores CPU leg: the unmodified oracle on several host threads, each on its own run of buckets.
    On a tiny workload held in host memory the changed elements it finds must be exactly those of the buckets it
    covered (taken from a single-threaded oracle run over the whole set)."""
    sys.path.insert(0, ROOT)
    import numpy as np
    import torch

    import bench
    import oracle
    from paper_2605_07330_amd import synth
    wl = synth.workload(2, tiny=True)
    a = synth.WeightSet(wl, "cpu", slab=False); b = synth.WeightSet(wl, "cpu", slab=False)
    synth.fill_base(a, 5)
    synth.make_update(b, a, 5)
    numels, be, nb = a.numels, wl.bucket_elems, wl.num_buckets
    _, _, counts, _ = oracle.extract_multi(a.to_numpy_u16(), b.to_numpy_u16(), numels, be)
    wall, elems, used, changed = bench.cpu_all_cores(torch, np, oracle, wl, a, b, cores=3, buckets_per_thread=2)
    assert used == min(3, nb // 2) and wall > 0
    stride = nb // used
    covered = [bk for c in range(used) for bk in range(c * stride, min(nb, c * stride + 2))]
    assert len(set(covered)) == len(covered), "the threads' bucket runs must not overlap"
    assert changed == int(counts[covered].astype(np.int64).sum())
    assert elems == sum(min(wl.numel, (bk + 1) * be) - bk * be for bk in covered)
    assert a.equal(a) and not a.equal(b), "the weight sets themselves are left alone (host copies are refreshed)"
