"""The C oracle built with AddressSanitizer and UndefinedBehaviorSanitizer (host code, CPU only) and the
whole pin suite run against that build: an out-of-bounds index, a use of uninitialised stack or a signed
overflow in the checker would otherwise go unnoticed as long as the numbers came out right."""
import os
import shutil
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parents[1]


def test_pin_suite_against_a_sanitizer_build(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not asan or not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc has no libasan here")
    src = tmp_path / "dvp_oracle_sanitized.c"
    shutil.copy(ROOT / "oracle" / "dvp_oracle.c", src)
    env = dict(os.environ)
    env["DVP_ORACLE_SRC"] = str(src)
    env["DVP_ORACLE_CFLAGS"] = "-g -fno-omit-frame-pointer -fsanitize=address,undefined -fno-sanitize-recover=all"
    # the sanitizer runtime has to come first among the preloaded libraries of the interpreter
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"       # the interpreter itself is not leak-clean
    res = subprocess.run([sys.executable, "-m", "pytest", str(ROOT / "tests" / "test_oracle_pins.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = res.stdout[-3000:] + res.stderr[-3000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
    assert (tmp_path / "dvp_oracle_sanitized.so").exists()          # the instrumented build is the one that ran
