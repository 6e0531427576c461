"""CPU checks of bench.py's bookkeeping: the HBM-traffic figure is only reported
while the committed counter summary was measured on the kernel sources in the
tree, and a request for more than one GPU is refused."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402


def test_traffic_figure_is_tied_to_the_kernel_sources(tmp_path, monkeypatch):
    h = bench.kernel_sources_hash()
    assert len(h) == 16 and h == bench.kernel_sources_hash()
    traffic, note = bench.traffic_from_profiles()
    assert note["kernel_sources"] == h and note["source"].startswith("profiles")
    if traffic is None:
        assert note.get("stale") or note.get("missing")
    else:
        assert note["measured_on_kernel_sources"] == h
        assert 0.95 < traffic / (18 * 134217728) < 1.10
    # a summary measured on other sources is not reported
    fake = tmp_path / "profiles"
    fake.mkdir()
    (fake / "reduce_n_allreduce_bf16_256MiB_pmc.txt").write_text(
        "kernel_sources_sha256: 0123456789abcdef\ntraffic_bytes_per_launch: 2415810981\n")
    real_root = bench.ROOT
    monkeypatch.setattr(bench, "kernel_sources_hash", lambda: h)
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    traffic, note = bench.traffic_from_profiles()
    assert traffic is None and note["stale"] is True
    (fake / "reduce_n_allreduce_bf16_256MiB_pmc.txt").write_text(
        "kernel_sources_sha256: %s\ntraffic_bytes_per_launch: 2415810981\n" % h)
    traffic, note = bench.traffic_from_profiles()
    assert traffic == 2415810981.0
    monkeypatch.setattr(bench, "ROOT", real_root)


def test_more_than_one_gpu_is_refused():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert run.returncode != 0 and "one GPU" in run.stderr
