"""bench.py command line without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_traffic_figure_is_only_reported_for_the_kernel_source_it_was_measured_on(tmp_path, monkeypatch):
    sys.path.insert(0, ROOT)
    import bench
    f = tmp_path / "traffic.txt"
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(f))
    assert bench.traffic_from_profile("h8192", "rank", "flat-bf16") == (None, None)        # no file
    sha = bench.kernel_source_hash()
    f.write_text(f"# comment\nh8192 rank flat-bf16 {sha} 1996407061 1.9999 0.9984 profiles/x.md\n"
                 f"h8192 group flat-bf16 {'0' * 16} 32294697052 1.9999 0.9986 profiles/y.md\n")
    value, source = bench.traffic_from_profile("h8192", "rank", "flat-bf16")
    assert value == 1996407061 and sha in source
    value, source = bench.traffic_from_profile("h8192", "group", "flat-bf16")              # other source hash
    assert value is None and source.startswith("stale")
    assert bench.traffic_from_profile("h4096", "rank", "flat-bf16") == (None, None)         # never measured
