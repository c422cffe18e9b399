"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no HIP): the library's
repacker and column-block quantizers and the C oracle are compiled with g++/gcc -fsanitize=address,undefined
into one program (tests/sanitize_driver.cpp) that runs every host entry point on ragged and extreme
shapes with exactly-sized heap buffers; any out-of-bounds access, misaligned access or undefined
arithmetic makes the program fail."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_04477_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="needs gcc and g++")
def test_host_sources_and_oracle_are_clean_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    obj = tmp_path / "oracle.o"
    exe = tmp_path / "sanitize_driver"
    subprocess.run(["gcc", "-std=c11", *san, "-fopenmp", "-c", "-o", str(obj), os.path.join(ROOT, "oracle", "spqt_oracle.c")],
                   check=True, capture_output=True, text=True)
    r = subprocess.run(["g++", "-std=c++17", *san, *inc, "-fopenmp", "-pthread", "-o", str(exe),
                        os.path.join(ROOT, "tests", "sanitize_driver.cpp"), os.path.join(CSRC, "pack.cpp"),
                        os.path.join(CSRC, "quant_cb.cpp"), str(obj), "-lm"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1",
               OMP_NUM_THREADS="2")
    env.pop("LD_PRELOAD", None)      # the sanitizer runtime must come first in the program's own link order
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "sanitize_driver: clean" in run.stdout
