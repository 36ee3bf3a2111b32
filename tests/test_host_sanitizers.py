"""The library's host code (renumbering, relabelling, transpose, weights, model) under ASan + UBSan,
and once more under TSan (the row-parallel passes use worker threads on large graphs).

Builds csrc/gnn_host.cpp with g++ and the sanitizers together with a small C++ driver and runs it:
memory errors, undefined behaviour or data races in the host-side preparation abort the driver."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
@pytest.mark.parametrize("sanitizers", ["address,undefined", "thread"])
def test_host_entry_points_are_clean_under_sanitizers(sanitizers):
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "host_sanitizer_driver")
        cmd = ["g++", "-std=c++17", "-O1", "-g", f"-fsanitize={sanitizers}", "-fno-sanitize-recover=all", "-pthread",
               "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2006_06608_amd", "csrc"),
               os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"),
               os.path.join(ROOT, "paper_2006_06608_amd", "csrc", "gnn_host.cpp"), "-o", exe]
        build = subprocess.run(cmd, capture_output=True, text=True)
        assert build.returncode == 0, build.stderr[-2000:]
        env = dict(os.environ)
        # a library preloaded into every process comes before the sanitizer runtime; that is fine here
        env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
        env["TSAN_OPTIONS"] = "halt_on_error=1"
        run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
        assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
        assert "ok" in run.stdout
