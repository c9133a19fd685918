"""The oracle's pins once more, on a build of oracle/sdtw_oracle.c with the address and
undefined-behaviour sanitizers (CPU only).

The interpreter itself is not instrumented, so the sanitizer runtime has to be preloaded into a
child process; that child re-runs tests/test_oracle_pins.py against ``libsdtw_oracle_san.so``
(``SDTW_ORACLE_SANITIZE=1``, see oracle/sdtw_oracle.py).  An out-of-bounds access, a use after
free or an undefined operation in the oracle aborts the child, which fails this test.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    path = subprocess.check_output(["gcc", "-print-file-name=" + name], text=True).strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_pins_under_sanitizers():
    asan, ubsan = _runtime("libasan.so"), _runtime("libubsan.so")
    if asan is None:
        pytest.skip("gcc has no libasan.so here")
    sys.path.insert(0, ROOT)
    import oracle

    lib = oracle.build(force=True, sanitize=True)
    assert os.path.exists(lib)
    env = dict(os.environ)
    env["SDTW_ORACLE_SANITIZE"] = "1"
    # the sanitizer runtime goes in front of whatever is preloaded already
    pre = [asan] + ([ubsan] if ubsan else []) + [p for p in env.get("LD_PRELOAD", "").split(":") if p]
    env["LD_PRELOAD"] = ":".join(pre)
    # leaks of the interpreter are not the oracle's; the link-order check would refuse a preload
    # that is not the first library of the process
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "2"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    tail = r.stdout[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in tail and "ERROR: AddressSanitizer" not in r.stdout and "runtime error:" not in r.stdout, tail
