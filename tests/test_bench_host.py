"""Host-side pieces of bench.py that need no GPU: the contract for more than one GPU, the algorithmic byte and
flop model behind the roofline figures, the stamp that ties a traffic record to the kernel sources, and the power
sampler's behaviour on a machine without the hwmon file."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from paper_2410_01623_amd import synth  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0
    assert "one GPU" in (p.stdout + p.stderr) or "1 GPU" in (p.stdout + p.stderr) or "single" in (p.stdout + p.stderr).lower()


def test_algorithmic_model_of_the_headline_workload():
    wl = synth.WORKLOADS[synth.HEADLINE]
    shapes = wl.shapes
    mn = sum(m * n for m, n in shapes)
    Lr = sum(max(m, n) * wl.rank for m, n in shapes)
    Sr = sum(min(m, n) * wl.rank for m, n in shapes)
    model = bench.kernel_models(shapes, wl.rank, "gram")
    # one contraction each: 2 mn r flops
    assert model["update"]["flops"] == pytest.approx(2.0 * mn * wl.rank)
    # update: G read, W read and written (2 bytes each), Z and P read once
    assert model["update"]["bytes"] == pytest.approx(6 * mn + 2 * Lr + 2 * Sr)
    fused = model["project"]["bytes"] + model["adam_norms"]["bytes"]
    assert fused >= 2 * mn + 16 * Lr           # at least G once and M, V read and written


def test_traffic_record_is_dropped_when_the_sources_changed(tmp_path, monkeypatch):
    stamp = bench.kernel_sources_hash()
    assert len(stamp) == 16
    prof = tmp_path / "profiles"
    prof.mkdir()
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    monkeypatch.setattr(bench, "kernel_sources_hash", lambda: stamp)
    (prof / "hbm_traffic_w_gram.txt").write_text(f"# kernel_sources {stamp}\nupdate 123\n")
    assert bench.read_traffic("w", "gram") == {"update": 123.0}
    (prof / "hbm_traffic_w_gram.txt").write_text("# kernel_sources 0000000000000000\nupdate 123\n")
    assert bench.read_traffic("w", "gram") == {}
    assert bench.read_traffic("missing", "gram") == {}


def test_power_sampler_without_the_hwmon_file(monkeypatch):
    import glob
    monkeypatch.setattr(glob, "glob", lambda pattern: [])
    with bench.PowerSampler() as ps:
        pass
    assert ps.mean() is None and ps.cap() is None
