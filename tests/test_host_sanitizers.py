"""The library's host-only sources (expert packing, the 12-bit form, the host cores' expert path with its worker
pool) built with the host sanitizers and run on a small case: AddressSanitizer + UndefinedBehaviorSanitizer in one
build, ThreadSanitizer in another, each on the instruction-set paths this machine has.  No GPU involved."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_20179_amd", "csrc")
SOURCES = [os.path.join(ROOT, "tests", "host_sanitize", "main.cpp"), os.path.join(CSRC, "host_experts.cpp"),
           os.path.join(CSRC, "host_pack.cpp")]


@pytest.mark.parametrize("name,flags", [("asan-ubsan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"]),
                                        ("tsan", ["-fsanitize=thread", "-static-libtsan"])])
def test_host_sources_under_sanitizers(tmp_path, name, flags):
    exe = str(tmp_path / ("host_sanitize_" + name))
    cmd = [os.environ.get("CXX", "g++"), "-O1", "-g", "-std=c++17", "-pthread", "-Wall", "-Wno-psabi", *flags,
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, *SOURCES, "-o", exe]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout
    for isa in ("", "avx2", "generic"):
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
                   TSAN_OPTIONS="halt_on_error=1")
        if isa:
            env["TIDE_HOST_ISA"] = isa
        run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
        assert run.returncode == 0 and "host sanitize ok" in run.stdout, "%s (isa %r):\n%s" % (name, isa or "native", run.stdout[-4000:])
