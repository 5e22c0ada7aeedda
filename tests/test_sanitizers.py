"""Address / undefined-behaviour sanitizer builds of the CPU-side code, run on the CPU: the oracle
(gcc) and the host paths of the C ABI (hipcc, sanitizers on the host side only, kernel variant tables
left empty so that no device code is needed).  A sanitizer report makes the drivers exit non-zero."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
CSRC = os.path.join(ROOT, "paper_2603_29010_amd", "csrc")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd[:4])} ... failed:\n{r.stdout[-2000:]}\n{r.stderr[-4000:]}"
    return r


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-g", "-std=c11", "-D_GNU_SOURCE", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
          "-fno-omit-frame-pointer", os.path.join(ROOT, "oracle", "ucl_oracle.c"), os.path.join(SAN, "oracle_driver.c"),
          "-o", exe, "-lm"])
    r = _run([exe], env=dict(ENV, OMP_NUM_THREADS="2"))
    assert "oracle sanitizer driver: ok" in r.stdout and "ERROR" not in r.stderr and "runtime error" not in r.stderr


def test_host_api_under_address_and_undefined_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not shutil.which(hipcc):
        pytest.skip("hipcc not found")
    # every instantiation unit's table, empty
    decls = re.findall(r"VariantList (variants_\w+)\(\);", open(os.path.join(CSRC, "ucl_variants.h")).read())
    stub = tmp_path / "empty_variants.cpp"
    stub.write_text('#include "ucl_variants.h"\nnamespace ucl {\n' +
                    "".join(f"VariantList {d}() {{ return {{nullptr, 0}}; }}\n" for d in decls) + "}\n")
    exe = str(tmp_path / "host_api_san")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
    _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-command-line-argument", "-x", "hip", *san, "-I", CSRC, "-I", os.path.join(ROOT, "include"),
          os.path.join(CSRC, "ucl_api.hip"), os.path.join(CSRC, "ucl_transpose.hip"), str(stub),
          os.path.join(SAN, "host_api_driver.cpp"), "-o", exe], cwd=str(tmp_path))
    r = _run([exe], env=ENV)
    assert "host API sanitizer driver: ok" in r.stdout and "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr
