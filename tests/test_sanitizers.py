"""CPU sanitizer job: the oracle (plain C) and the host side of the C-ABI library (cache index, argument checks of the
context calls) are built with AddressSanitizer + UndefinedBehaviorSanitizer into stand-alone drivers
(tests/sanitize/*) and run as child processes.  Only HOST code is instrumented (-fno-gpu-sanitize on the hipcc lines);
no device is touched: the drivers call nothing that reaches the HIP runtime."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-3000:]}\n{r.stderr[-3000:]}"
    return r


def _clean(r):
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr and "LeakSanitizer" not in r.stderr, r.stderr[-3000:]


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-std=c99", "-fopenmp", *SAN, "-static-libasan", os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-o", exe, "-lm"])
    r = _run([exe], env=ENV)
    _clean(r)
    assert "oracle driver: ok" in r.stdout


def test_cache_index_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "host_driver")
    _run(["g++", "-std=c++17", "-I" + os.path.join(ROOT, "include"), *SAN, "-static-libasan",
          os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"),
          os.path.join(ROOT, "paper_2601_11553_amd", "csrc", "cache_tree.cpp"), "-o", exe])
    r = _run([exe], env=ENV)
    _clean(r)
    assert "host driver: ok" in r.stdout


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
def test_abi_host_layer_under_address_and_ub_sanitizers(tmp_path):
    """The whole library, host code instrumented, linked with the driver: config validation, the refusals of
    percache_create (bad shape, NULL / misaligned / short arena) and the NULL-context paths run without a device."""
    from paper_2601_11553_amd.build import CSRC, FLAGS, HIPCC, SOURCES
    hip_san = SAN + ["-fno-gpu-sanitize", "-Wno-pass-failed"]
    flags = [f for f in FLAGS if f != "-O3"]

    def compile_one(src):
        obj = str(tmp_path / (os.path.splitext(src)[0] + ".o"))
        _run([HIPCC, *flags, *hip_san, "-c", os.path.join(CSRC, src), "-o", obj])
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    drv = str(tmp_path / "driver.o")
    _run([HIPCC, *flags, *hip_san, "-DWITH_CONTEXT", "-x", "hip", "-c", os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"), "-o", drv])
    exe = str(tmp_path / "host_driver_ctx")
    _run([HIPCC, "--offload-arch=gfx950", *hip_san, drv, *objs, "-o", exe])
    r = _run([exe], env=ENV)
    _clean(r)
    assert "host driver: ok" in r.stdout
