"""The CPU checker under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): rs_oracle.c
is compiled with a small driver that calls every routine on exactly sized heap buffers and ragged
sizes; any out-of-bounds access, use of freed memory, signed overflow or misaligned access aborts it."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("openmp", [False, True])
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path, openmp):
    if shutil.which("gcc") is None:
        pytest.skip("gcc not available")
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", os.path.join(ROOT, "oracle", "rs_oracle.c"),
           os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c"), "-o", exe, "-lm"]
    if openmp:
        cmd.insert(1, "-fopenmp")
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and "asan" in (r.stderr + r.stdout).lower() and "cannot find" in (r.stderr + r.stdout).lower():
        pytest.skip("sanitizer runtime not installed")
    assert r.returncode == 0, r.stderr
    env = dict(os.environ)
    # other preloaded libraries may come before the sanitizer runtime: do not insist on the link order
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, (r.stdout, r.stderr)
    assert r.stdout.strip() == "ok"
