"""CPU-only checks of bench.py's host logic: the stored HBM-traffic figures are only reported while the
HIP sources hash to the value they were measured with, and more than one GPU is refused."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_traffic_figures_are_tied_to_the_source_hash(monkeypatch):
    sys.path.insert(0, ROOT)
    import bench
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    assert os.path.exists(path)
    stamped = [ln.split()[1] for ln in open(path) if ln.startswith("source_sha256")]
    assert len(stamped) == 1 and len(stamped[0]) == 64
    # whatever the stamp says, figures come back exactly when the running sources hash to it
    monkeypatch.setattr(bench, "source_hash", lambda: stamped[0])
    for workload in ("room115k", "scene1p2m", "batch16x60k"):
        t = bench.measured_traffic(workload)
        assert set(t) == set(bench.KERNEL_KEYS) and all(v > 0 for v in t.values())
    assert bench.measured_traffic("no_such_workload") == {}
    monkeypatch.setattr(bench, "source_hash", lambda: "0" * 64)
    assert bench.measured_traffic("room115k") == {}          # other sources: the figures would be stale


def test_source_hash_covers_every_hip_source(tmp_path, monkeypatch):
    sys.path.insert(0, ROOT)
    import bench
    h0 = bench.source_hash()
    assert h0 == bench.source_hash() and len(h0) == 64
    src = os.path.join(ROOT, "paper_2103_15076_amd", "csrc")
    names = sorted(n for n in os.listdir(src) if n.endswith((".h", ".hip")))
    assert "picasso.hip" in names and "primitives.h" in names and "decimate_kernels.h" in names
    # a copy of the tree with one byte more in one header hashes differently
    root2 = tmp_path / "r"
    (root2 / "paper_2103_15076_amd" / "csrc").mkdir(parents=True)
    for n in names:
        data = open(os.path.join(src, n), "rb").read()
        (root2 / "paper_2103_15076_amd" / "csrc" / n).write_bytes(data + (b"\n" if n == "pooling.h" else b""))
    monkeypatch.setattr(bench, "ROOT", str(root2))
    assert bench.source_hash() != h0


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)
