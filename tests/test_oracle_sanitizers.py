"""The oracle under the host sanitizers: oracle/sanitize_main.c drives every entry point of oracle/slicemoe_oracle.c on
small layers with exactly-sized buffers, built with -fsanitize=address,undefined (CPU only; GPU code is not involved)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    src = [os.path.join(ROOT, "oracle", n) for n in ("sanitize_main.c", "slicemoe_oracle.c")]
    build = subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined",
                            "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", exe, *src, "-lm"],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ)
    # whatever the environment preloads stays: the link-order check is relaxed instead
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "sanitize_main: ok" in run.stdout
    assert "ERROR" not in run.stderr and "runtime error" not in run.stderr, run.stderr
