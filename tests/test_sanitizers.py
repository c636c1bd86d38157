"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host code, run on the CPU:
  * the whole oracle (oracle/int8t_oracle.c) on small ragged cases, with gcc;
  * the host side of the C-ABI layer (csrc/api.hip: argument checks, size queries, host plans, the
    code-unpacking aid), with hipcc's host pass instrumented and the device code left alone.  Every
    call in the driver returns before a launch, so no GPU is needed.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
CSRC = os.path.join(ROOT, "paper_1912_12607_amd", "csrc")


def run_clean(exe):
    p = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=300)
    text = p.stdout.decode(errors="replace")
    assert p.returncode == 0, text
    assert "AddressSanitizer" not in text and "runtime error" not in text, text
    return text


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    subprocess.run(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-ffp-contract=off",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan",
                    "-o", exe, os.path.join(SAN, "oracle_sanitize_driver.c"), "-lm"], check=True)
    assert "oracle sanitize ok" in run_clean(exe)


def test_abi_host_paths_under_asan_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc")
    from paper_1912_12607_amd import build as b
    b.build(force=False)                       # the other object files, as built for the library
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    api_o = str(tmp_path / "api_san.o")
    subprocess.run([hipcc] + b.FLAGS + san + ["-g", "-c", os.path.join(CSRC, "api.hip"), "-o", api_o], check=True)
    drv_o = str(tmp_path / "drv.o")
    subprocess.run([hipcc, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                    "-fno-gpu-sanitize", "-x", "c++", "-c", os.path.join(SAN, "abi_sanitize_driver.cpp"), "-o", drv_o], check=True)
    objs = [os.path.join(CSRC, s.replace(".hip", ".o")) for s in b.SOURCES if s != "api.hip"]
    exe = str(tmp_path / "abi_sanitize")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize",
                    "-o", exe, drv_o, api_o] + objs, check=True)
    assert "abi sanitize ok" in run_clean(exe)
