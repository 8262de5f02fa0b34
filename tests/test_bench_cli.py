"""Host-only checks of bench.py's command line (no GPU)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_world_size_above_one_is_refused_too():
    env = dict(os.environ, WORLD_SIZE="4", RANK="0")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True,
                       timeout=120, env=env)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_traffic_table_points_at_existing_sources():
    sys.path.insert(0, ROOT)
    import bench
    for rec in bench.MEASURED_TRAFFIC.values():
        for name in rec["sources"]:
            assert os.path.exists(os.path.join(ROOT, "paper_2405_01943_amd", "csrc", name)), name
        assert len(rec["sha256"]) == 64 and rec["bytes"] > 0
