"""CPU sanitizer tier: the oracle's C source and the library's host boundary (descriptor validation and expansion,
slot placement, the scheduler's arithmetic) built with AddressSanitizer + UndefinedBehaviorSanitizer and driven
with valid, malformed and randomly mutated inputs by the programs under tests/sanitize/.  No GPU: the kernel
launchers the boundary calls are stubbed out in the driver."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2601_11546_amd", "csrc")
SAN_DIR = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-3000:]}\n{r.stderr[-3000:]}"
    return r.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
          "-fno-omit-frame-pointer", "-I", os.path.join(ROOT, "oracle"), os.path.join(ROOT, "oracle", "relserve_oracle.c"),
          os.path.join(SAN_DIR, "oracle_driver.c"), "-o", exe, "-lm"])
    assert "ok" in _run([exe], env=ENV)


def test_sanitizer_build_reports_a_planted_overrun(tmp_path):
    """The same flags on a program that reads one element past a heap buffer: the build must catch it, otherwise the
    two green runs beside this test would mean nothing."""
    src = tmp_path / "overrun.c"
    src.write_text("#include <stdlib.h>\nint main(int argc, char** argv) { int* p = (int*)malloc(8 * sizeof(int)); "
                   "for (int i = 0; i < 8; ++i) p[i] = i; int s = p[7 + argc]; free(p); return s == 12345; }\n")
    exe = str(tmp_path / "overrun")
    _run(["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", str(src), "-o", exe])
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV)
    assert r.returncode != 0 and ("heap-buffer-overflow" in r.stderr or "insufficient space" in r.stderr)


def test_host_boundary_under_asan_ubsan(tmp_path):
    san = []
    for flag in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"):
        san += ["-Xarch_host", flag]                        # host side only: no device sanitizer on this pool
    common = ["hipcc", "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-fno-gpu-rdc", "-Xclang", "-target-feature", "-Xclang",
              "-packed-fp32-ops", *san, "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = []
    for name in ("relserve_api", "duration_model"):
        objs.append(str(tmp_path / f"{name}.o"))
        _run([*common, "-c", os.path.join(CSRC, f"{name}.hip"), "-o", objs[-1]])
    objs.append(str(tmp_path / "host_driver.o"))
    _run([*common, "-x", "hip", "-c", os.path.join(SAN_DIR, "host_driver.cpp"), "-o", objs[-1]])
    exe = str(tmp_path / "host_san")
    _run(["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", *objs, "-o", exe])
    out = _run([exe], env=ENV)
    assert "ok" in out and "400 valid descriptors" in out
