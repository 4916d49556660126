"""The host code of the library (packer, reference quantizer, blob queries) and the CPU oracle, built
with AddressSanitizer and UndefinedBehaviorSanitizer and run on small matrices (CPU only; the GPU
code is not part of this build)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_packer_quantizer_and_oracle_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "sanitize_main"
    obj = tmp_path / "oracle.o"
    flags = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
    subprocess.run(["gcc", "-std=c11", "-ffp-contract=off", "-fopenmp", *flags, "-c",
                    os.path.join(ROOT, "oracle", "mpq_oracle.c"), "-o", str(obj)], check=True)
    subprocess.run(["g++", "-std=c++17", "-ffp-contract=off", "-fopenmp", *flags, "-static-libasan",   # the runtime inside the executable: no ordering requirement on preloaded libraries
                   
                    os.path.join(ROOT, "tests", "sanitize_main.cpp"),
                    os.path.join(ROOT, "paper_2311_16442_amd", "csrc", "mpq_pack.cpp"), str(obj), "-lm", "-o", str(exe)],
                   check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    if "runtime does not come first" in run.stderr:
        pytest.skip("the environment preloads a library in front of the sanitizer runtime")
    assert run.returncode == 0 and run.stdout.strip().endswith("ok"), (run.returncode, run.stdout[-2000:], run.stderr[-4000:])
