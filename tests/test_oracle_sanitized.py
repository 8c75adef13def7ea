"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (host only, no GPU involved).

pc_oracle.c is compiled once more with -fsanitize=address,undefined and every pin of test_oracle_pins.py is run
against that build in a child process (the sanitizer runtime has to be loaded before the interpreter starts).
An out-of-bounds index, a read of freed memory, a signed overflow or a misaligned access anywhere the pins reach
ends the child with a report.
"""
import os
import subprocess
import sys
import tempfile

import oracle

_CHILD = r"""
import sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import oracle
oracle._load()
oracle._lib = oracle._bind({lib!r})          # every oracle call of this process now runs the instrumented build
import pytest
sys.exit(pytest.main(["-q", "-x", "-p", "no:cacheprovider", {pins!r}]))
"""


def _runtime(name: str) -> str:
    return subprocess.run(["gcc", f"-print-file-name={name}"], check=True, capture_output=True, text=True).stdout.strip()


def test_pins_pass_on_an_asan_ubsan_build_of_the_oracle():
    tests = os.path.dirname(os.path.abspath(__file__))
    root = os.path.dirname(tests)
    asan, ubsan = _runtime("libasan.so"), _runtime("libubsan.so")
    assert os.path.isabs(asan) and os.path.isabs(ubsan), "the host compiler ships no sanitizer runtime"
    with tempfile.TemporaryDirectory() as td:
        lib = os.path.join(td, "libpc_oracle_san.so")
        subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fsanitize=address,undefined",
                        "-fno-sanitize-recover=undefined", "-o", lib, oracle._SRC, "-lm"], check=True)
        env = dict(os.environ)
        preload = [asan, ubsan] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else [])
        env["LD_PRELOAD"] = ":".join(preload)
        env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0"      # the interpreter's own allocations are not the subject
        code = _CHILD.format(root=root, tests=tests, lib=lib, pins=os.path.join(tests, "test_oracle_pins.py"))
        r = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=600)
    report = r.stdout[-3000:] + r.stderr[-3000:]
    assert "AddressSanitizer" not in report and "runtime error:" not in report, report
    assert r.returncode == 0, report
    assert " passed" in r.stdout, report
