"""The C of the oracle and the host half of the library, rebuilt with AddressSanitizer and UBSan and driven on
the CPU (no GPU needed).  Device code is not part of these builds: the host half is compiled host-only and linked
against tests/sanitize/hip_stub.hip, whose launchers launch nothing and instead check on the host what their
kernels assume; memory the host code copies to or from is real memory of exactly the size the library asks for."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT = os.path.join(ROOT, "_build", "sanitize")
SAN = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-3000:]}\n{r.stderr[-6000:]}"
    return r


def test_oracle_under_sanitizers():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_check")
    _run(["gcc", *SAN, "-static-libasan", "-static-libubsan", "-fopenmp", os.path.join(ROOT, "oracle", "alaya_oracle.c"),
          os.path.join(ROOT, "tests", "sanitize", "oracle_check.c"), "-lm", "-o", exe])
    r = _run([exe], env=ENV)
    assert "oracle_check: 0 failures" in r.stdout


def test_library_host_side_under_sanitizers():
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    clangxx = "/opt/rocm/llvm/bin/clang++"
    if not (os.path.exists(hipcc) and os.path.exists(clangxx)):
        pytest.skip("no hipcc / clang++ here")
    os.makedirs(OUT, exist_ok=True)
    csrc = os.path.join(ROOT, "paper_2504_10326_amd", "csrc")
    objs = []
    for src in (os.path.join(csrc, "api.hip"), os.path.join(csrc, "plan.hip"), os.path.join(ROOT, "tests", "sanitize", "hip_stub.hip")):
        obj = os.path.join(OUT, os.path.basename(src) + ".o")
        _run([hipcc, "--offload-host-only", "-std=c++17", *SAN, "-c", src, "-o", obj])
        objs.append(obj)
    drv = os.path.join(OUT, "host_check.o")
    _run([clangxx, "-std=c++17", *SAN, "-I/opt/rocm/include", "-c", os.path.join(ROOT, "tests", "sanitize", "host_check.cpp"), "-o", drv])
    # a host-only object still refers to the device image that it would have carried; nothing here reads it
    undefined = subprocess.run(["nm", "-u", *objs], capture_output=True, text=True).stdout
    fatbins = sorted({w for w in undefined.split() if w.startswith("__hip_fatbin_")})
    exe = os.path.join(OUT, "host_check")
    _run([clangxx, *SAN, *objs, drv, *[f"-Wl,--defsym={s}=0" for s in fatbins], "-o", exe])
    r = _run([exe], env=ENV)
    assert "host_check: 0 failures, 0 launch-check failures" in r.stdout
