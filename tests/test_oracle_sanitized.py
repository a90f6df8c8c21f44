"""The oracle's pins once more, against a build of tdfa_oracle.c with AddressSanitizer and
UndefinedBehaviorSanitizer (host code only; nothing here touches a GPU).  The pins run in a child
process that has the sanitizer's runtime preloaded; any report ends that process with an error."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["test_oracle_compile.py", "test_oracle_mask.py", "test_oracle_advance.py", "test_oracle_terminals.py",
             "test_oracle_minimize.py", "test_oracle_compact.py", "test_oracle_sample.py", "test_oracle_pda.py"]


@pytest.mark.skipif(os.environ.get("TDFA_ORACLE_SANITIZE") == "1", reason="already inside the sanitized run")
def test_oracle_pins_under_asan_ubsan():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc has no libasan here")
    env = dict(os.environ)
    env["TDFA_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter itself is not instrumented: its own allocations are not this test's business
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    files = [os.path.join(ROOT, "tests", f) for f in PIN_FILES if os.path.exists(os.path.join(ROOT, "tests", f))]
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout, tail
