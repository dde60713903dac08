"""Host-side safety net: the page bookkeeping of the paged KV cache (csrc/pages.h, the host-only part
of the library's allocator) built for the CPU with AddressSanitizer and UndefinedBehaviorSanitizer and
driven through reserve / roll back / share / exhaust sequences; the row packing of partial stages is checked there too
(tests/host/pages_driver.cpp)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_page_bookkeeping_under_sanitizers(tmp_path):
    exe = str(tmp_path / "pages_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-I", os.path.join(ROOT, "paper_2501_19324_amd", "csrc"), os.path.join(ROOT, "tests", "host", "pages_driver.cpp"),
           "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "pages ok" in r.stdout
