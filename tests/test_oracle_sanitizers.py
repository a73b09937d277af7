"""The CPU checker's C code under AddressSanitizer and UndefinedBehaviorSanitizer (host side only):
a small C driver calls every exported function on ragged shapes with exactly-sized buffers."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE = os.path.join(os.path.dirname(HERE), "oracle")
SRC = [os.path.join(HERE, "sanitize", "oracle_sanitize_main.c"), os.path.join(ORACLE, "dn_oracle.c"),
       os.path.join(ORACLE, "dn_conv_oracle.c")]


@pytest.mark.parametrize("store,prefix", [("float", "o32_"), ("double", "o64_")])
def test_checker_is_clean_under_asan_and_ubsan(tmp_path, store, prefix):
    exe = str(tmp_path / ("oracle_sanitize_" + store))
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-DSTORE_T=" + store, "-DPFX(x)=" + prefix + "##x", *SRC, "-o", exe, "-lm"]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="2")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    sys.stderr.write(run.stderr[-2000:])
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "sanitize ok" in run.stdout
