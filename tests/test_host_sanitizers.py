"""AddressSanitizer + UndefinedBehaviorSanitizer on the host code: the CPU oracle (every function,
on small problems with exactly sized buffers) and the host pass of the HIP library (argument
validation, block planning, workspace sizing, knobs, profiler bookkeeping; no kernel is launched).
Needs no GPU.  Sanitizers run on host code only."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "host_sanitize")
OUT = os.path.join(HERE, "_build")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")


def run(cmd, **kw):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    return proc.returncode, proc.stdout


def assert_clean(rc, out, what):
    for marker in ("AddressSanitizer", "runtime error", "UndefinedBehaviorSanitizer", "FAILED"):
        assert marker not in out, (what, out[-4000:])
    assert rc == 0, (what, rc, out[-4000:])


def test_oracle_under_asan_ubsan():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_driver")
    rc, out = run(["gcc", "-std=c99", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined",
                   "-fno-sanitize-recover=undefined", "-static-libasan", "-o", exe,
                   os.path.join(HERE, "oracle_driver.c"), os.path.join(ROOT, "oracle", "lory_oracle.c"), "-lm"])
    assert rc == 0, out
    rc, out = run([exe], env=ENV)
    print(out)
    assert_clean(rc, out, "oracle")
    assert "oracle sanitizer run: ok" in out


@pytest.mark.timeout(900)
def test_library_host_layer_under_asan_ubsan():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    os.makedirs(OUT, exist_ok=True)
    csrc = os.path.join(ROOT, "paper_2405_03133_amd", "csrc")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-gpu-rdc",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
             "-w", "-I", os.path.join(ROOT, "include"), "-I", csrc] + san
    srcs = sorted(glob.glob(os.path.join(csrc, "*.hip")))
    procs = []
    objs = []
    for src in srcs:
        obj = os.path.join(OUT, os.path.basename(src)[:-4] + ".san.o")
        objs.append(obj)
        procs.append((src, subprocess.Popen([hipcc] + flags + ["-c", src, "-o", obj], stdout=subprocess.PIPE,
                                            stderr=subprocess.STDOUT, text=True)))
    for src, pr in procs:
        out, _ = pr.communicate()
        assert pr.returncode == 0, (src, out[-4000:])
    drv = os.path.join(OUT, "abi_driver.san.o")
    rc, out = run([hipcc] + flags + ["-x", "hip", "-c", os.path.join(HERE, "abi_driver.cpp"), "-o", drv])
    assert rc == 0, out[-4000:]
    exe = os.path.join(OUT, "abi_driver")
    rc, out = run([hipcc, "--offload-arch=gfx950", "-fno-gpu-rdc", "-fsanitize=address", "-fsanitize=undefined",
                   "-fno-gpu-sanitize"] + objs + [drv, "-o", exe])
    assert rc == 0, out[-4000:]
    rc, out = run([exe], env=ENV)
    print(out)
    assert_clean(rc, out, "abi")
    assert "abi sanitizer run: ok" in out
    shutil.rmtree(OUT, ignore_errors=True)
