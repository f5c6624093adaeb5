"""Host sanitizer build of the oracle: oracle/fwa_oracle.c and a small C driver compiled with
AddressSanitizer and UndefinedBehaviorSanitizer, run in a subprocess on two small shapes (and an
empty batch) through every entry point; any report makes the process exit non-zero."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc on this machine")
    exe = str(tmp_path / "oracle_asan")
    # the sanitizer runtimes are linked statically: a dynamically linked ASan refuses to start in a
    # process that already has another preloaded library in front of it
    cmd = [gcc, "-O1", "-g", "-std=c99", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-static-libasan", "-static-libubsan", "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "oracle", "fwa_oracle.c"), os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
           "-lm"]
    built = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if built.returncode != 0 and ("asan" in built.stdout.lower() or "ubsan" in built.stdout.lower()
                                  or "sanitize" in built.stdout.lower()):
        pytest.skip("this gcc has no sanitizer runtime to link: " + built.stdout.strip().splitlines()[-1])
    assert built.returncode == 0, built.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0 and "clean" in run.stdout, run.stdout[-4000:]
    assert "ERROR: AddressSanitizer" not in run.stdout and "runtime error" not in run.stdout, run.stdout[-4000:]
