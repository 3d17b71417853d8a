"""The host translation unit of the library (threaded SVD with a hand-written barrier and spin-wait, rank schedule,
index helpers) built with gcc's sanitizers and run on a driver that checks its results: AddressSanitizer +
UndefinedBehaviorSanitizer in one build, ThreadSanitizer in another.  CPU only; the GPU sources are not involved."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = [os.path.join(ROOT, "paper_2410_03111_amd", "csrc", "lorc_host.cpp"), os.path.join(ROOT, "tests", "host_sanitize_main.cpp")]
INC = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2410_03111_amd", "csrc")]


@pytest.mark.parametrize("name,flags", [
    ("asan_ubsan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan"]),
    ("tsan", ["-fsanitize=thread", "-static-libtsan"]),
])
def test_host_library_under_sanitizers(tmp_path, name, flags):
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / f"host_{name}")
    build = subprocess.run([cxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-pthread", *flags, *INC, *SRC, "-o", exe],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    env = dict(os.environ, LORC_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1", TSAN_OPTIONS="halt_on_error=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "0 failed checks" in run.stdout
