"""bench.py's command line where no GPU is needed: more than one GPU is refused with a message, and
the digest that ties the stored HBM-traffic counters to the kernel sources matches the sources."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], cwd=ROOT,
                       capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "one gpu" in (r.stdout + r.stderr).lower() or "single" in (r.stdout + r.stderr).lower()
    assert not r.stdout.strip().startswith("{")


def test_traffic_digest_is_well_formed():
    sys.path.insert(0, ROOT)
    import bench
    assert len(bench.csrc_digest()) == 64
    assert bench.HBM_TRAFFIC["batch"] == 32 and bench.HBM_TRAFFIC["fetch_bytes"] > 0 and bench.HBM_TRAFFIC["write_bytes"] > 0
