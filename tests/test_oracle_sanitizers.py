"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/fier_oracle.c compiled together with a
small C driver (tests/sanitize/oracle_driver.c) that calls every oracle function on the edge shapes -- empty and
one-token sequences, lengths around a group boundary, partial tail groups, group sizes 32 / 128 / 256, budgets above
the length and above the row pitch, appends into an empty cache, pages without tokens -- with every buffer allocated
at exactly its size.  Any access past an end or undefined arithmetic aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan",
           os.path.join(ROOT, "oracle", "fier_oracle.c"), os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
           "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    # (the sanitizer runtime is linked statically, so whatever the environment preloads does not disturb it)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.strip() == "ok", r.stdout + r.stderr
