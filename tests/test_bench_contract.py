"""Host-side contract of bench.py and the entry module (no GPU needed)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_bench_refuses_a_multi_rank_launch():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True,
                       timeout=120, env=env)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_traffic_files_parse_and_are_tied_to_the_kernel_sources(tmp_path, monkeypatch):
    sys.path.insert(0, ROOT)
    import bench
    assert bench.read_traffic("no_such_workload")[0] is None
    prof = os.path.join(ROOT, "profiles")
    names = [f[len("traffic_"):-4] for f in os.listdir(prof) if f.startswith("traffic_") and f.endswith(".txt")]
    assert names
    for name in names:
        v, note = bench.read_traffic(name)
        # a summary is either current (a figure) or reported stale (no figure, the reason given)
        assert (v is not None and v > 1e6) or "stale" in note, (name, note)
    # a summary stamped with other kernel sources is not used
    monkeypatch.setattr(bench, "kernel_source_sha", lambda names=None: "0" * 16)
    for name in names:
        v, note = bench.read_traffic(name)
        assert v is None and "stale" in note


def test_bench_defaults_to_the_largest_single_gpu_configuration():
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert '"--config", type=int, default=4' in src


def test_entry_module_has_build_and_smoke():
    sys.path.insert(0, ROOT)
    import __graft_entry__ as g
    assert callable(g.build) and callable(g.smoke)


def test_gpu_marker_is_registered():
    ini = open(os.path.join(ROOT, "pytest.ini")).read() if os.path.exists(os.path.join(ROOT, "pytest.ini")) else ""
    conf = open(os.path.join(ROOT, "tests", "conftest.py")).read()
    assert "gpu" in ini or "gpu" in conf
