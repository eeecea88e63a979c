"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU call is made).

1. The C oracle: tests/san/oracle_driver.c calls every oracle function on heap buffers of exactly the
   documented sizes, so an index that strays by one element trips ASan.
2. The library's host side: every source of the C-ABI library is compiled with its HOST pass instrumented
   (device code untouched) and tests/san/abi_driver.cpp walks argument validation, options, error text and the
   context life cycle on a context without a device.
"""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "san")
BAD = ("ERROR: AddressSanitizer", "runtime error:", "ERROR: LeakSanitizer")


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    out = r.stdout + r.stderr
    assert not any(b in out for b in BAD), out[-4000:]
    assert r.returncode == 0, out[-4000:]
    return out


def test_oracle_under_asan_ubsan(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_san")
    subprocess.run(["gcc", "-std=c99", "-O1", "-g", "-fopenmp", "-ffp-contract=off",
                    "-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-o", exe,
                    os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "clada_oracle.c"), "-lm"],
                   check=True, capture_output=True, text=True)
    assert "0 failures" in _run(exe)


def test_library_host_code_under_asan_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    csrc = os.path.join(ROOT, "paper_2502_19078_amd", "csrc")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", csrc]
    san_host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-omit-frame-pointer"]
    procs = []
    for src in sorted(glob.glob(os.path.join(csrc, "*.hip"))):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        procs.append((src, obj, subprocess.Popen(
            [hipcc, "-c", src, "-o", obj, *inc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *san_host],
            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for src, obj, p in procs:
        log, _ = p.communicate(timeout=1200)
        assert p.returncode == 0, f"{src}:\n{log[-3000:]}"
        objs.append(obj)
    drv = str(tmp_path / "abi_driver.o")
    subprocess.run([hipcc, "-std=c++17", "-O1", "-g", *inc, "-fsanitize=address,undefined", "-fno-gpu-sanitize",
                    "-c", os.path.join(SAN, "abi_driver.cpp"), "-o", drv], check=True, capture_output=True, text=True)
    exe = str(tmp_path / "abi_san")
    subprocess.run([hipcc, "-fsanitize=address,undefined", "-fno-gpu-sanitize", "--offload-arch=gfx950",
                    "-o", exe, drv, *objs], check=True, capture_output=True, text=True)
    assert "0 failures" in _run(exe)
