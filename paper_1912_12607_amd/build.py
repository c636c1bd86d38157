"""Builds csrc/libint8t.so (the C-ABI HIP library) for gfx950 with hipcc.

hipcc cross-compiles without a GPU.  Flags: no fused multiply-add contraction (the fp32
arithmetic that decides an int8 code must round exactly as stated in include/int8t.h), and the
compiler's automatic packed-fp32 instruction selection switched off.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(CSRC, "libint8t.so")
SOURCES = ["api.hip", "quantize.hip", "dsgc.hip", "conv_igemm.hip", "conv_band.hip", "conv_wgrad.hip", "conv_wgrad_lines.hip", "s2d.hip", "conv_dw.hip", "profile.hip"]
HEADERS = ["device_common.h", "kernels.h", "profile.h", "lds_dma.h", os.path.join("..", "..", "include", "int8t.h")]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-fno-fast-math", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]
# Per-file additions.  dsgc.hip: keep the MFMA accumulators in ordinary vector registers (the kernel
# has registers to spare); otherwise the compiler parks them in accumulation registers and copies
# all of them back and forth on every trip of the inner loop.
EXTRA_FLAGS = {"dsgc.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _stale(obj: str, deps) -> bool:
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    hdrs = [os.path.join(CSRC, h) for h in HEADERS]
    objs = []
    procs = []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(CSRC, src.replace(".hip", ".o"))
        objs.append(o)
        if force or _stale(o, [s] + hdrs):
            cmd = [hipcc] + FLAGS + EXTRA_FLAGS.get(src, []) + ["-c", s, "-o", o]
            if verbose:
                print(" ".join(cmd), flush=True)
            procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        text = out.decode(errors="replace")
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"--- hipcc failed on {src} ---\n{text}\n")
        elif verbose and text.strip():
            print(text)
    if failed:
        raise RuntimeError("hipcc failed")
    if force or procs or not os.path.exists(LIB):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
