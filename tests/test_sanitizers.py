"""Host sanitizer builds (no GPU): the CPU oracle and the host half of the library (argument
checks, host packing, the profile linear program) are compiled with AddressSanitizer and
UndefinedBehaviorSanitizer on the HOST side only and driven by small programs under
tests/sanitize/.  Device code is compiled as usual and never runs here.  Objects are cached under
paper_2605_18856_amd/_build_asan (rebuilt when a source changes)."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2605_18856_amd import build as libbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT = os.path.join(ROOT, "paper_2605_18856_amd", "_build_asan")
ENV = dict(os.environ, ASAN_OPTIONS="abort_on_error=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _run(exe, env):
    p = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    text = p.stdout
    assert p.returncode == 0, text[-4000:]
    assert "AddressSanitizer" not in text and "runtime error:" not in text, text[-4000:]
    return text


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    gcc = shutil.which("gcc")
    if not gcc:
        pytest.skip("no host C compiler")
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_asan")
    srcs = [os.path.join(ROOT, "oracle", "bsse_oracle.c"), os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c")]
    if _stale(exe, srcs):
        subprocess.run([gcc, "-std=c11", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined",
                        "-fno-sanitize-recover=all"] + srcs + ["-lm", "-o", exe], check=True)
    assert "ok" in _run(exe, ENV)


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers():
    hipcc = libbuild.HIPCC
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    os.makedirs(OUT, exist_ok=True)
    # host-side sanitizers only: each -fsanitize option rides on its own -Xarch_host
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]
    flags = [f for f in libbuild.FLAGS if f != "-O3"] + ["-O1", "-g"] + san
    jobs, objs = [], []
    for src in libbuild.SOURCES:
        s = os.path.join(libbuild.CSRC, src)
        o = os.path.join(OUT, src.replace(".hip", ".o"))
        objs.append(o)
        if _stale(o, [s] + libbuild.HEADERS + [os.path.join(libbuild.CSRC, "gen_device.h")]):
            jobs.append([hipcc] + flags + ["-c", s, "-o", o])
    drv_src = os.path.join(ROOT, "tests", "sanitize", "abi_driver.cpp")
    drv = os.path.join(OUT, "abi_driver.o")
    if _stale(drv, [drv_src] + libbuild.HEADERS):
        jobs.append([hipcc, "-std=c++17", "-O1", "-g", "-x", "hip", "--offload-arch=gfx950"] + san + ["-c", drv_src, "-o", drv])
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        list(ex.map(lambda c: subprocess.run(c, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL), jobs))
    exe = os.path.join(OUT, "abi_asan")
    if jobs or _stale(exe, objs + [drv]):
        subprocess.run([hipcc, "--offload-arch=gfx950"] + san + ["-o", exe] + objs + [drv], check=True,
                       stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    # (the HIP runtime's own start-up allocations are not this library's to free)
    env = dict(ENV, ASAN_OPTIONS="abort_on_error=0:detect_leaks=0")
    assert "ok" in _run(exe, env)
