"""The CPU side under AddressSanitizer and UndefinedBehaviorSanitizer.

The oracle's C cores (oracle_core.c, grow_core.c) and the input generator's grower (forest_grower.cpp) are rebuilt with
-fsanitize=address,undefined, and the CPU test files that exercise them run again in a child process that has the
sanitizer runtimes preloaded; any report ends that run with an error.  CPU only: nothing of this touches a GPU."""
import os
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parents[1]
FILES = ["tests/test_oracle_counts.py", "tests/test_oracle_factors.py", "tests/test_oracle_grow.py",
         "tests/test_oracle_consumers.py", "tests/test_inputs.py"]


def _runtime(name):
    out = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


def test_oracle_and_input_generator_under_sanitizers():
    if os.environ.get("RFX_SANITIZE") == "1":
        pytest.skip("already inside the sanitized run")
    asan, ubsan = _runtime("libasan.so"), _runtime("libubsan.so")
    if not asan or not ubsan:
        pytest.skip("gcc's sanitizer runtimes are not installed")
    env = dict(os.environ)
    env.update({
        "RFX_SANITIZE": "1",
        "LD_PRELOAD": " ".join(filter(None, [asan, ubsan, env.get("LD_PRELOAD", "")])),
        # python itself leaks by design; link order is not checked because the interpreter is not instrumented
        "ASAN_OPTIONS": "detect_leaks=0:verify_asan_link_order=0:halt_on_error=1:abort_on_error=0",
        "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1",
        "OMP_NUM_THREADS": "4",
    })
    r = subprocess.run([sys.executable, "-m", "pytest", *FILES, "-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    assert " passed" in r.stdout
