"""The host-side argument checks of the C ABI under AddressSanitizer and
UndefinedBehaviorSanitizer: the library is built once more with the sanitizers on the HOST
side only (device code is compiled as usual and never runs here) and the CPU-only ABI tests
are run against that build in a child process.  Any report ends the child with an error."""
import os
import subprocess
import sys

import pytest

from paper_2407_01378_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT_DIR = os.path.join(ROOT, "_build")
SAN_LIB = os.path.join(OUT_DIR, "libthc_hostsan.so")

CHILD = """
import sys
sys.path.insert(0, {root!r})
import paper_2407_01378_amd.binding as b
b.LIB_PATH = {lib!r}
import pytest
sys.exit(pytest.main(["-q", "-x", "-s", "-p", "no:cacheprovider", {tests!r}]))
"""


def _asan_runtime():
    hipcc = build.command("x")[0]
    res = subprocess.run([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE,
                         stderr=subprocess.DEVNULL, text=True)
    path = res.stdout.strip()
    return path if res.returncode == 0 and os.path.isabs(path) and os.path.exists(path) else None


def test_abi_host_checks_under_host_sanitizers():
    runtime = _asan_runtime()
    if runtime is None:
        pytest.skip("this toolchain ships no shared AddressSanitizer runtime")
    os.makedirs(OUT_DIR, exist_ok=True)
    cmd = [a for a in build.command(SAN_LIB) if a != "-O3"] + [
        "-O1", "-g",
        "-Xarch_host", "-fsanitize=address",
        "-Xarch_host", "-fsanitize=undefined",
        "-Xarch_host", "-fno-sanitize-recover=undefined"]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    env = dict(os.environ)
    # the sanitizer runtime has to come first among the loaded libraries of the child (python
    # itself is not instrumented); whatever is preloaded already stays, after it
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    tests = os.path.join(ROOT, "tests", "test_abi_host.py")
    child = subprocess.run([sys.executable, "-c", CHILD.format(root=ROOT, lib=SAN_LIB, tests=tests)],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    tail = child.stdout[-4000:]
    assert child.returncode == 0, tail
    assert "runtime error" not in child.stdout and "AddressSanitizer" not in child.stdout, tail
    assert " passed" in child.stdout, tail
