"""The oracle and the library's host-side code (argument checks, workspace layouts, launch tables, split
plans) built with -fsanitize=address,undefined and run on the CPU.  Device code is not sanitized (no GPU
sanitizer runs on this pool); the drivers under tests/sanitize/ never launch a kernel."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout[-2000:]}\n{res.stderr[-4000:]}"
    return res


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
          "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan", "-static-libubsan", "-Wall", "-Wextra",
          "-o", exe, os.path.join(SAN, "oracle_main.c"), os.path.join(ROOT, "oracle", "dsv_oracle.c"), "-lm"])
    out = _run([exe], env=ENV)
    assert "oracle sanitizer run ok" in out.stdout


def test_library_host_code_under_address_and_undefined_sanitizers(tmp_path):
    sys.path.insert(0, ROOT)
    from paper_2502_07590_amd.build import CSRC, HIPCC_FLAGS, SOURCES, _hipcc
    from concurrent.futures import ThreadPoolExecutor
    hipcc = _hipcc()
    # each -fsanitize goes to the host pass only (directly after -Xarch_host); device code is built as always
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-g"]
    flags = [f for f in HIPCC_FLAGS if f != "-O3"] + ["-O1"]

    def compile_one(src):
        obj = str(tmp_path / (src + ".o"))
        _run([hipcc, *flags, *san, "-c", os.path.join(CSRC, src), "-o", obj])
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    main_o = str(tmp_path / "main.o")
    _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", *san, "-I", os.path.join(ROOT, "include"), "-c",
          "-x", "c++", os.path.join(SAN, "host_checks_main.cpp"), "-o", main_o])
    exe = str(tmp_path / "host_san")
    _run([hipcc, "--offload-arch=gfx950", *san, "-o", exe, main_o, *objs])
    out = _run([exe], env=ENV)
    assert "host checks sanitizer run ok" in out.stdout
