"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a small
C driver (tests/sanitize_oracle.c) calls every entry point of oracle/bigmac_oracle.c on ragged
shapes with exactly sized heap buffers; any out-of-bounds access, use after free, leak, signed
overflow or misaligned access fails the run."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_oracle")
    cmd = ["gcc", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-mavx2", "-mfma", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra", "-o", exe,
           os.path.join(HERE, "sanitize_oracle.c"), os.path.join(ROOT, "oracle", "bigmac_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert p.returncode == 0 and p.stdout.strip().endswith("ok"), p.stdout[-4000:]
