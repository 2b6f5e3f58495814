"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a small driver (oracle_sanitize_main.cpp) that
calls every entry point on ragged and degenerate inputs is compiled together with the oracle's source and run as a
process of its own, with the sanitizer runtimes linked statically.  CPU only."""
import os
import shutil
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_oracle_runs_clean_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-fno-omit-frame-pointer", os.path.join(HERE, "oracle_sanitize_main.cpp"), os.path.join(ROOT, "oracle", "floe_oracle.cpp"),
           "-lpthread", "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    env = dict(os.environ)          # (the sanitizer runtimes are linked statically: nothing has to be preloaded)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    sys.stdout.write(run.stdout)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "oracle sanitizer run: ok" in run.stdout
