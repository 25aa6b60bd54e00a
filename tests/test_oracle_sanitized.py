"""The CPU oracle under the host sanitizers: oracle/dit_oracle.c and a small C driver are built
with -fsanitize=address,undefined and run; any out-of-bounds access, leak of an index past a
buffer, signed overflow or misaligned access inside the oracle aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-o", exe, os.path.join(ROOT, "oracle", "dit_oracle.c"),
           os.path.join(ROOT, "tests", "oracle_sanitize_main.c"), "-lm"]
    subprocess.check_call(cmd)
    # (verify_asan_link_order=0: the process may carry preloaded libraries ahead of the sanitizer runtime)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0", OMP_NUM_THREADS="4")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout
    assert "0 failure(s)" in r.stdout, r.stdout
