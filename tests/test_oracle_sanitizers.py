"""The oracle's C code under AddressSanitizer + UndefinedBehaviorSanitizer (host only, small inputs)."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_c_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-fast-math", "-ffp-contract=off", os.path.join(ROOT, "oracle", "fnn_oracle.c"),
           os.path.join(HERE, "oracle_sanitizer_main.c"), "-lm", "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "sanitizer" in build.stderr.lower():
        pytest.skip("this gcc has no sanitizer runtime: " + build.stderr[-200:])
    assert build.returncode == 0, build.stderr
    env = {k: v for k, v in os.environ.items() if k != "LD_PRELOAD"}   # ASan insists on being first in the list
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.strip() == "ok"
