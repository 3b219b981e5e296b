"""The host half of the library - inspector, code generator, plan persistence, the C boundary -
built with g++ -fsanitize=address,undefined and driven through a grid of problems in a native
process (tests/host_sanitize/main.cpp; the device half is replaced by stubs that refuse).
A memory error or undefined behaviour anywhere in that code fails this test, on the CPU, before
a kernel built from the same arithmetic ever reaches a GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2008_11849_amd", "csrc")
HERE = os.path.join(ROOT, "tests", "host_sanitize")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-static-libubsan", "-I", os.path.join(ROOT, "include"), "-o", exe,
           os.path.join(HERE, "main.cpp"), os.path.join(HERE, "stubs.cpp")]
    cmd += [os.path.join(CSRC, f) for f in ("api.cpp", "inspect.cpp", "specialize.cpp", "serialize.cpp")]
    cmd += ["-ldl", "-lpthread"]
    build = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert build.returncode == 0, build.stderr[-3000:]
    # leaks are reported for this build's own code only: the code object manager keeps
    # process-lifetime state of its own
    supp = tmp_path / "lsan.supp"
    supp.write_text("leak:libamd_comgr\nleak:libLLVM\n")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               LSAN_OPTIONS=f"suppressions={supp}:print_suppressions=0")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "0 failed expectations" in run.stdout
