"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU-side code, run as part of the CPU
suite: the fp64 oracle (gcc) through tests/sanitize/oracle_driver.c, and the library's host logic --
csrc/sn_api.hip (argument checks, workspace queries, planner) and csrc/sn_runtime.cpp (pool, route,
memory traces) compiled with host-side sanitizers -- through tests/sanitize/host_driver.cpp, linked
with the library's other objects.  Nothing here launches a kernel or needs a GPU; device code is
not instrumented (host flags only)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT = os.path.join(ROOT, "tests", "sanitize", "_build")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, "%s\n%s" % (" ".join(cmd), r.stdout[-4000:])
    return r.stdout


def test_oracle_under_asan_ubsan():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_driver")
    _run(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
          "-fno-sanitize-recover=undefined", "-o", exe, os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
          os.path.join(ROOT, "oracle", "sn_oracle.c"), "-lm"])
    out = _run([exe], env=ENV)
    assert "oracle driver: ok" in out


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc builds the host side of the .hip sources")
def test_library_host_logic_under_asan_ubsan():
    from paper_1801_04380_amd import build
    build.build_library()          # the other translation units' objects, as the library has them
    os.makedirs(OUT, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    objs = []
    for name in ("sn_api.hip", "sn_runtime.cpp"):
        obj = os.path.join(OUT, name + ".san.o")
        _run(["hipcc"] + [f for f in build.FLAGS if f != "-O3"] + ["-O1", "-g"] + san +
             ["-c", os.path.join(build.CSRC, name), "-o", obj])
        objs.append(obj)
    drv = os.path.join(OUT, "host_driver.o")
    _run(["hipcc", "-O1", "-g", "-std=c++17", "-I", os.path.join(ROOT, "include")] + san +
         ["-c", os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"), "-o", drv])
    others = [os.path.join(build.OBJ, f) for f in sorted(os.listdir(build.OBJ))
              if f.endswith(".o") and not f.startswith(("sn_api.", "sn_runtime."))]
    exe = os.path.join(OUT, "host_driver")
    _run(["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", exe, drv] + objs + others)
    out = _run([exe], env=ENV)
    assert "host driver: ok" in out
