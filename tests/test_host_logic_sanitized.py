"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no kernel is launched).

Every source is compiled once more with the sanitizers on the host pass (`-Xarch_host -fsanitize=...`; device code
is compiled as always) and the GPU-free checks of test_abi_host.py (exported symbols, schema layout, uncached
positions, selection and overlap checks, scaffold resolution, bytes per token) are run against that build in a child
process: the sanitizer runtime has to be loaded before the interpreter starts.
"""
import glob
import os
import subprocess
import sys
import tempfile

from paper_2311_04934_amd import build as pc_build

_CHILD = r"""
import sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import paper_2311_04934_amd.build as bb
import paper_2311_04934_amd.binding as b
bb.ensure_built = lambda: {lib!r}
b.LIB_PATH = {lib!r}                      # every library call of this process now runs the instrumented build
import pytest
sys.exit(pytest.main(["-q", "-x", "-p", "no:cacheprovider", {target!r}]))
"""


def test_host_checks_pass_on_an_asan_ubsan_build_of_the_library():
    tests = os.path.dirname(os.path.abspath(__file__))
    root = os.path.dirname(tests)
    rts = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    assert rts, "the HIP compiler ships no sanitizer runtime"
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = [f for f in pc_build.FLAGS if f != "-O3"] + ["-O1", "-g"]
    with tempfile.TemporaryDirectory() as td:
        objs, procs = [], []
        for src in pc_build.SOURCES:
            objs.append(os.path.join(td, src.replace(".hip", ".o")))
            procs.append(subprocess.Popen([pc_build.HIPCC, *flags, *san, "-c", os.path.join(pc_build.CSRC, src), "-o", objs[-1]],
                                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
        for p in procs:
            out, _ = p.communicate()
            assert p.returncode == 0, out[-3000:]
        lib = os.path.join(td, "libpromptcache_san.so")
        subprocess.run([pc_build.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                        "-shared-libsan", "-o", lib, *objs], check=True, capture_output=True)
        env = dict(os.environ)
        env["LD_PRELOAD"] = ":".join([rts[0]] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else []))
        env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0"      # the interpreter's own allocations are not the subject
        code = _CHILD.format(root=root, tests=tests, lib=lib, target=os.path.join(tests, "test_abi_host.py"))
        r = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=600)
    report = r.stdout[-3000:] + r.stderr[-3000:]
    assert "AddressSanitizer" not in report and "runtime error:" not in report, report
    assert r.returncode == 0, report
    assert " passed" in r.stdout, report
