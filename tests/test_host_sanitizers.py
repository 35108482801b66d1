"""The host side of the library (csrc/knap_host.c: topology parser, greedy balancer, chunking, model fit)
compiled with AddressSanitizer and UndefinedBehaviorSanitizer into a small fuzz driver and run on seeded
random and degenerate inputs: malformed strings, empty bags, zero weights, zero capacities, undersized
output arrays.  Host code only; no GPU and no HIP compiler involved."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
def test_host_code_is_clean_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "host_fuzz")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-Wall", "-Wextra", "-Werror",
           "-I" + os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "host_fuzz_driver.c"),
           os.path.join(ROOT, "paper_2508_06001_amd", "csrc", "knap_host.c"),
           "-lm", "-o", exe]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "host fuzz ok" in run.stdout
