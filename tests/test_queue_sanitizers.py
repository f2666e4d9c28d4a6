"""The non-blocking task queue (section 3.2 of the paper) under the host sanitizers: the stress program
tests/native/queue_stress.cpp is built with g++ -fsanitize=thread and -fsanitize=address,undefined and
must run clean (every id exactly once, per-producer order, no report from the sanitizer) with a node
pool far smaller than the id count, so that every node is recycled thousands of times."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("san", ["thread", "address,undefined"])
@pytest.mark.parametrize("n,p,c,cap", [(150000, 3, 3, 64), (60000, 1, 4, 2), (60000, 4, 1, 1000)])
def test_queue_stress_is_clean(tmp_path, san, n, p, c, cap):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "queue_stress")
    build = subprocess.run([gxx, "-std=c++17", "-O1", "-g", "-fsanitize=" + san, "-fno-omit-frame-pointer",
                            "-I", os.path.join(ROOT, "paper_1511_04348_amd", "csrc"),
                            os.path.join(ROOT, "tests", "native", "queue_stress.cpp"), "-o", exe, "-lpthread"],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if build.returncode != 0 and ("cannot find" in build.stdout or "unrecognized" in build.stdout):
        pytest.skip("sanitizer runtime not installed: " + build.stdout[-200:])
    assert build.returncode == 0, build.stdout
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1", ASAN_OPTIONS="detect_leaks=1", UBSAN_OPTIONS="halt_on_error=1")
    run = subprocess.run([exe, str(n), str(p), str(c), str(cap)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, timeout=300, env=env)
    assert run.returncode == 0, run.stdout[-2000:]
    assert run.stdout.startswith("ok:") and "Sanitizer" not in run.stdout, run.stdout[-2000:]
