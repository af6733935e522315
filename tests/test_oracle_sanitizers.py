"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a small driver calls
every entry on seeded cases with exactly sized heap buffers, including empty active sets, k larger than a
set, an empty batch union, clusters that lose their members, recorded tokens outside the vocabulary and
missing beam candidates."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCES = ["vp_oracle.c", "vp_train_oracle.c", "vp_search_oracle.c"]


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = tmp_path / "oracle_sanitize"
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", os.path.join(ROOT, "tests", "oracle_sanitize_main.c")]
    cmd += [os.path.join(ROOT, "oracle", s) for s in SOURCES] + ["-lm", "-o", str(exe)]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle sanitizer run ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr
