"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer.

The oracle is the root of every parity claim and does raw pointer arithmetic over strided layouts, so it is
compiled once more with `-fsanitize=address,undefined` together with tests/sanitize/oracle_driver.c, which calls
every entry point on buffers allocated at exactly the size the call may touch: padded heads, slots and rows,
`n_src` below what is allocated, indices without a source slot, the in-place path with `n_keep = n_src - 1`,
selections with `k = 0`, `M = k + 1`, `n_recent = 0`, the LM-head score with padded leading dimensions, serial and
threaded.  A clean exit with no sanitizer report is the result."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.timeout(300)
def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    assert gcc, "gcc is part of this image"
    exe = tmp_path / "oracle_sanitized"
    cmd = [gcc, "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra",
           "-I", os.path.join(ROOT, "oracle"), os.path.join(ROOT, "oracle", "sirllm_ref.c"),
           os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-lm", "-o", str(exe)]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    env.pop("LD_PRELOAD", None)                      # the sanitizer runtime must come first in the link order
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=240)
    report = (run.stdout + "\n" + run.stderr)[-4000:]
    assert run.returncode == 0, report
    assert "SANITIZED OK" in run.stdout, report
    assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error:" not in run.stderr, report
