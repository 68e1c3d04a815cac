"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only; no GPU).

A small C driver (tests/csrc/oracle_sanitizer_driver.c) calls every entry point of oracle/kgc_oracle.c on seeded
inputs with exactly-sized and too-short output buffers; both files are compiled into one executable with
-fsanitize=address,undefined (runtime linked statically, so that nothing has to be preloaded) and run once.  A
heap overflow, a leak of a result list, a signed overflow or a misaligned access in the oracle fails the test."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan", "-o", exe,
           os.path.join(HERE, "csrc", "oracle_sanitizer_driver.c"), os.path.join(ROOT, "oracle", "kgc_oracle.c"), "-lm"]
    built = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if built.returncode != 0 and ("asan" in built.stdout.lower() or "sanitize" in built.stdout.lower()):
        pytest.skip("this gcc has no sanitizer runtime: " + built.stdout.strip().splitlines()[-1])
    assert built.returncode == 0, built.stdout
    env = dict(os.environ)
    env["OMP_NUM_THREADS"] = "4"
    # (OpenMP's own thread pool is not freed at exit: that is not the oracle's leak)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["LSAN_OPTIONS"] = "suppressions=" + os.path.join(HERE, "csrc", "lsan.supp")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout
    assert run.stdout.strip().endswith("ok"), run.stdout
    assert "runtime error" not in run.stdout and "AddressSanitizer" not in run.stdout, run.stdout
