"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

oracle/selfcheck.c drives both oracle files over a few shapes; any out-of-bounds access, use of
uninitialised heap through the sanitizer's poisoning, leak or undefined arithmetic fails the run.
"""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_sanitizers(tmp_path):
    exe = str(tmp_path / "selfcheck")
    src = [os.path.join(ROOT, "oracle", f) for f in ("selfcheck.c", "sig_oracle.c", "sig_grad_oracle.c")]
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-ffp-contract=off", "-o", exe] + src + ["-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "sanitize" in built.stderr:
        pytest.skip("this gcc has no sanitizer runtime: " + built.stderr.splitlines()[-1])
    assert built.returncode == 0, built.stderr
    # (verify_asan_link_order=0: the process may run with other preloaded libraries ahead of the sanitizer runtime)
    env = dict(os.environ, OMP_NUM_THREADS="2",
               ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    ran = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert ran.returncode == 0, ran.stdout + ran.stderr
    assert "selfcheck ok" in ran.stdout
