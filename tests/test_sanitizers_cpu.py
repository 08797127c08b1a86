"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the code that executes on the host: the
library's boundary (argument checks, plan and workspace arithmetic, the host side of the
hand-off) and the column-wise CPU sampler.  No GPU is used: the library is built host-only (its
device code left out, an empty offload bundle standing in for it) and every call the driver
makes is one the host rejects or answers by itself.  The drivers are tests/sanitize/*.

The enum check of UBSan is off for the library: its C boundary takes enum parameters from C
callers, which may hand over any int, and validates them itself."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-O1", "-g"]


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if "is not a recognized feature" not in l)
    return res.returncode, out


def test_columnwise_cpu_sampler_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if not gcc:
        pytest.skip("no gcc")
    exe = str(tmp_path / "cw_san")
    rc, out = _run([gcc, "-std=gnu11", *SAN, "-static-libasan", "-fopenmp",
                    os.path.join(ROOT, "tests", "sanitize", "cw_main.c"), "-lm", "-o", exe])
    assert rc == 0, out
    rc, out = _run([exe], env={**os.environ, "ASAN_OPTIONS": "detect_leaks=1", "OMP_NUM_THREADS": "3"})
    assert rc == 0 and "ok" in out and "ERROR" not in out and "runtime error" not in out, out


def test_host_boundary_under_asan_and_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    clang = "/opt/rocm/lib/llvm/bin/clang"
    if not (os.path.exists(hipcc) and os.path.exists(clang)):
        pytest.skip("no hipcc / clang")
    lib = str(tmp_path / "libsip_san.so")
    rc, out = _run([hipcc, "--cuda-host-only", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
                    "-ffp-contract=off", *SAN, "-fno-sanitize=enum", "-I", os.path.join(ROOT, "include"), "-o", lib,
                    os.path.join(ROOT, "paper_2506_22033_amd", "csrc", "sip.hip")], cwd=str(tmp_path))
    assert rc == 0, out
    # the host code registers a device-code bundle that a host-only build does not contain:
    # give it one with no entries
    rc, syms = _run(["nm", "-D", "-u", lib])
    m = re.search(r"__hip_fatbin_[0-9a-f]+", syms)
    assert m, syms
    stub = tmp_path / "bundle_stub.cpp"
    stub.write_text("struct Bundle { char magic[24]; unsigned long long n; };\n"
                    "extern \"C\" { extern const Bundle %s; }\n"
                    "alignas(4096) const Bundle %s = {{'_','_','C','L','A','N','G','_','O','F','F','L','O','A','D','_',"
                    "'B','U','N','D','L','E','_','_'}, 0};\n" % (m.group(0), m.group(0)))
    exe = str(tmp_path / "boundary_san")
    rc, out = _run([clang + "++", "-std=c++17", *SAN, "-fno-sanitize=enum", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "sanitize", "boundary_main.cpp"), str(stub),
                    "-o", exe, "-L", str(tmp_path), "-lsip_san", "-Wl,-rpath," + str(tmp_path),
                    "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-lpthread"])
    assert rc == 0, out
    rc, out = _run([exe], env={**os.environ, "ASAN_OPTIONS": "detect_leaks=0"})
    assert rc == 0 and "ok" in out and "ERROR" not in out and "runtime error" not in out, out
