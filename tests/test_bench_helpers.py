"""Host-side pieces of bench.py that run without a GPU: progress lines never touch stdout (which carries the one
JSON record), the traffic record in profiles/ is tied to the kernel sources it was measured on, and more than
one GPU is refused with a message."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_progress_goes_to_stderr_only(capsys):
    import bench
    bench.progress("a step is done")
    out = capsys.readouterr()
    assert out.out == ""
    assert "a step is done" in out.err and out.err.startswith("# [")


def test_traffic_record_follows_the_kernel_sources(tmp_path, monkeypatch):
    import bench
    sha = bench.kernel_sources_sha()
    assert len(sha) == 64 and sha == bench.kernel_sources_sha()
    rec = os.path.join(ROOT, "profiles", "cfg3_target_gate_up_hbm_traffic.txt")
    fields = dict(l.strip().split("=", 1) for l in open(rec) if "=" in l and " " not in l.strip())
    got = bench.measured_traffic("cfg3")
    if fields["kernel_source_sha256"] == sha:
        assert got == int(fields["traffic_bytes_per_launch"]) and got > 0
    else:
        assert got is None                      # counters taken on other sources are not reported
    assert bench.measured_traffic("no_such_workload") is None
    # a changed kernel source withdraws the figure
    real = bench.kernel_sources_sha
    monkeypatch.setattr(bench, "kernel_sources_sha", lambda: "0" * 64)
    assert bench.measured_traffic("cfg3") is None
    monkeypatch.setattr(bench, "kernel_sources_sha", real)


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert p.stdout.strip() == ""
    assert "one GPU" in p.stderr
