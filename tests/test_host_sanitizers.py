"""Sanitizer tier for the host code (no GPU): every source of libplora is compiled again with AddressSanitizer and
UndefinedBehaviorSanitizer (and, in a second build, ThreadSanitizer with eight host threads) on its host side, linked with a small C++ driver (host_sanitize_driver.cpp) that walks
random valid and broken descriptions through every host-only entry point, through the argument checks of the device
entry points (each call fails its last check, so nothing is enqueued) and through the planner.  The run must end with
"ok" and without a sanitizer report.  Device code is not instrumented (the sanitizers are host-only here)."""
import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2508_02932_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST_SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
            "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def build_and_run(san_compile, san_link, args, env_extra):
    work = tempfile.mkdtemp(prefix="plora_san_")
    try:
        with ThreadPoolExecutor(max_workers=8) as ex:
            objs = list(ex.map(lambda s: build._compile(s, work, tuple(san_compile)), build.SOURCES))
        exe = os.path.join(work, "driver")
        drv = os.path.join(work, "driver.o")
        cmd = ["hipcc", "--offload-arch=gfx950", "-std=c++17", "-O1", *san_compile, "-I", os.path.join(ROOT, "include"),
               "-c", os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"), "-o", drv]
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-3000:]
        cmd = ["hipcc", "--offload-arch=gfx950", *san_link, "-fno-gpu-sanitize", "-pthread", drv, *objs, "-o", exe]
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-3000:]
        env = dict(os.environ, **env_extra)
        env.pop("LD_PRELOAD", None)
        run = subprocess.run([exe, *args], capture_output=True, text=True, env=env, timeout=900)
        if run.returncode != 0 and "unexpected memory mapping" in run.stderr:
            pytest.skip("the sanitizer runtime cannot map its shadow memory on this kernel (address-space layout), nothing ran")
        assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
        assert run.stdout.strip().startswith("ok "), run.stdout
        assert "Sanitizer" not in run.stderr and "runtime error" not in run.stderr, run.stderr[-4000:]
    finally:
        shutil.rmtree(work, ignore_errors=True)


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")
def test_host_code_under_asan_and_ubsan():
    build_and_run(HOST_SAN, ["-fsanitize=address", "-fsanitize=undefined"], ["300"],
                  dict(ASAN_OPTIONS="detect_leaks=0:halt_on_error=1", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1"))


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")
def test_host_code_under_tsan_with_eight_threads():
    tsan = ["-Xarch_host", "-fsanitize=thread", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    build_and_run(tsan, ["-fsanitize=thread"], ["60", "threads"], dict(TSAN_OPTIONS="halt_on_error=1:report_signal_unsafe=0"))
