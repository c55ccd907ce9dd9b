"""The CPU oracle's C source under the host sanitizers: rnn_oracle.c and a small C driver
(tests/oracle_sanitize_main.c) are compiled with -fsanitize=address,undefined and the driver runs two
of the oracle's pins (zero-weight closed form; central finite differences for every parameter of
a token/softmax-CE and a dense/tanh/MSE network).  An out-of-bounds index, a read of freed or
uninitialised-size memory, signed overflow or a misaligned access in the oracle ends the program
with a report instead of passing silently."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_pins_run_clean_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fopenmp", "-o", exe,
           os.path.join(HERE, "oracle_sanitize_main.c"), os.path.join(ROOT, "oracle", "rnn_oracle.c"), "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "asan" in (built.stderr or "").lower() and "cannot find" in built.stderr.lower():
        pytest.skip("the sanitizer runtime is not installed: " + built.stderr.strip().splitlines()[-1])
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, OMP_NUM_THREADS="2",
               ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.strip().endswith("ok"), run.stdout + run.stderr
    assert "ERROR" not in run.stderr and "runtime error" not in run.stderr, run.stderr
