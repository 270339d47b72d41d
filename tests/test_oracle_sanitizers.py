"""Host sanitizer pass: the C oracle under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU).

oracle/sanitize_check.c drives every entry point of oracle/scfa_oracle.c with small seeded inputs that cover
the method's edge cases; the program is built here with -fsanitize=address,undefined (the runtime linked
statically, so nothing has to be preloaded) and must exit 0 without a sanitizer report."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    src = [os.path.join(ROOT, "oracle", n) for n in ("sanitize_check.c", "scfa_oracle.c")]
    build = subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-std=c11", "-Wall", "-Wextra", "-Werror",
                            "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
                            "-o", exe, *src, "-lm"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "invariants hold" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
