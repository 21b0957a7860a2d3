"""The host side of the library (argument validation and dispatch in api.cpp, the block map and the plan
queries in blockmap.cpp, both on plan.h) built with AddressSanitizer and UndefinedBehaviorSanitizer and run
through tests/host_sanitize/driver.cpp: every entry point's refusal paths, the host-only size and state
functions, block maps and walk plans with result arrays of exactly the documented size.  The sanitizers
instrument host code only (the device code objects are the ordinary ones); no kernel is launched."""
import os
import shutil
import subprocess

import pytest

from paper_2509_15763_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
       "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
HOST_SOURCES = ["api.cpp", "blockmap.cpp"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout}\n{r.stderr}"
    return r


def test_host_code_under_asan_and_ubsan():
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    objdir = os.path.join(ROOT, "_build")
    device_objs = [os.path.join(objdir, os.path.splitext(s)[0] + ".o") for s in B.SOURCES if s not in HOST_SOURCES]
    if not all(os.path.exists(o) for o in device_objs):
        B.build_library()
    sandir = os.path.join(objdir, "host_sanitize")
    os.makedirs(sandir, exist_ok=True)
    objs = []
    for src in HOST_SOURCES:
        obj = os.path.join(sandir, os.path.splitext(src)[0] + ".o")
        _run([hipcc, *B.FLAGS, *SAN, "-c", os.path.join(B.CSRC, src), "-o", obj])
        objs.append(obj)
    drv = os.path.join(sandir, "driver.o")
    _run([hipcc, "-O1", "-std=c++17", "-x", "c++", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
          "-fno-omit-frame-pointer", "-g", "-I", os.path.join(ROOT, "include"), "-c",
          os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp"), "-o", drv])
    exe = os.path.join(sandir, "driver")
    _run([hipcc, "--offload-arch=gfx950", "-fno-gpu-sanitize", "-fsanitize=address,undefined", drv, *objs, *device_objs,
          "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0 and r.stdout.startswith("ok "), f"{r.stdout}\n{r.stderr[-4000:]}"
    assert int(r.stdout.split()[1]) > 1000
