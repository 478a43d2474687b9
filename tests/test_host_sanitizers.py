"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

tests/host_checks/driver.cpp calls the host-only helpers with ordinary, extreme and invalid
arguments and the argument validation of every device entry point; it is linked with the
library's sources, host side instrumented (the device code is compiled as usual and never
runs).  A sanitizer report or a failed expectation fails the test."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2510_17505_amd import _build

HERE = os.path.dirname(os.path.abspath(__file__))
OUT = os.path.join(_build.OBJ, "host_san")
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
       "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
       # the driver passes dtype codes outside the enum on purpose (the library must reject them,
       # and does so after converting to int): that load is what -fsanitize=enum would report
       "-Xarch_host", "-fno-sanitize=enum"]
FLAGS = [f if f != "-O3" else "-O1" for f in _build.HIPCC_FLAGS] + ["-g0"]


def _compile(src):
    path = src if os.path.isabs(src) else os.path.join(_build.CSRC, src)
    obj = os.path.join(OUT, os.path.splitext(os.path.basename(src))[0] + ".o")
    headers = [os.path.join(_build.CSRC, f) for f in os.listdir(_build.CSRC) if f.endswith(".h")]
    headers.append(os.path.join(_build.ROOT, "include", "insum.h"))
    newest = max(os.path.getmtime(f) for f in [path, __file__, *headers])
    if os.path.exists(obj) and os.path.getmtime(obj) > newest:
        return obj            # this object is up to date
    cmd = [_build._hipcc(), "-x", "hip", *FLAGS, *SAN, "-c", path, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, f"hipcc failed for {src}:\n{res.stderr[-3000:]}"
    return obj


@pytest.mark.timeout(900)
def test_host_code_under_asan_and_ubsan():
    os.makedirs(OUT, exist_ok=True)
    sources = list(_build.SOURCES) + [os.path.join(HERE, "host_checks", "driver.cpp")]
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(_compile, sources))
    exe = os.path.join(OUT, "host_checks")
    res = subprocess.run([_build._hipcc(), "--offload-arch=gfx950", *SAN, "-o", exe, *objs],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    report = run.stdout[-2000:] + run.stderr[-6000:]
    assert run.returncode == 0 and "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, report
    assert "host checks ok" in run.stdout
