"""Host-only sanitizer runs (AddressSanitizer + UBSan): the fp64 oracle on small inputs through every
entry point, and the host side of libclimber (argument validation, handles, workspace sizes) on calls
that return before any launch.  Both are built as stand-alone executables; no GPU is involved."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    return r.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-O1", "-g", "-fopenmp", "-std=c99", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-o", exe, os.path.join(SAN, "oracle_driver.c"), "-lm"])
    out = run([exe], env=dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1"))
    assert "rc=0" in out


def test_host_layer_under_asan_ubsan(tmp_path):
    from paper_2502_09888_amd import build as hb
    hipcc = hb._hipcc()
    csrc = hb.CSRC
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"]
    flags = [f for f in hb.FLAGS if f != "-fPIC"]
    objs = []
    procs = []
    for name in hb.SOURCES:
        obj = str(tmp_path / name.replace(".hip", ".o"))
        objs.append(obj)
        procs.append(subprocess.Popen([hipcc, *flags, *san, "-c", os.path.join(csrc, name), "-o", obj],
                                      stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True))
    for p in procs:
        out, err = p.communicate(timeout=600)
        assert p.returncode == 0, err[-3000:]
    exe, main_o = str(tmp_path / "host_san"), str(tmp_path / "host_driver.o")
    run(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-c", os.path.join(SAN, "host_driver.cpp"),
         "-o", main_o])
    run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", exe,
         main_o, *objs])
    # leak detection off: the HIP runtime keeps process-lifetime allocations of its own
    out = run([exe], env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"))
    assert "bad=0" in out
