"""Compile the HIP sources into paper_2510_08318_amd/liblinattn.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblinattn.so")
PROBE_LIB = os.path.join(HERE, "libmembw_probe.so")      # bench.py's streaming-rate probe, a library of its own
PROBE_SOURCE = "membw_probe.hip"
SOURCES = ["api.cpp", "fwd_f32.hip", "fwd_bf16.hip", "state_reduce.hip", "bwd_bf16.hip", "bwd_f32.hip", "relu_bf16.hip"]
# Packed-fp32 VALU forms are switched off for every device compilation.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]
# Per-file extras.  bwd_bf16.hip: MFMA results go to ordinary registers where they fit instead of
# always to the accumulation registers (the query-side backward kernel uses all 512 registers of a
# lane and spent a quarter of its vector instructions moving results between the two files:
# 149 -> 134 us at the config-5 shape; neutral or slightly worse for the other files).
EXTRA = {"bwd_bf16.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for src in SOURCES + [PROBE_SOURCE]:
        obj = os.path.join(HERE, "_build", src.rsplit(".", 1)[0] + ".o")
        cmd = [hipcc, *FLAGS, *EXTRA.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        if src.endswith(".cpp"):
            cmd.insert(1, "-x"); cmd.insert(2, "hip")
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if src != PROBE_SOURCE:
            objs.append(obj)
        else:
            probe_obj = obj
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        lines = [l for l in out.splitlines() if "not a recognized feature" not in l]
        if pr.returncode != 0:
            failed = True
            sys.stderr.write(f"[build] {src} FAILED\n" + "\n".join(lines) + "\n")
        elif verbose and lines:
            sys.stderr.write(f"[build] {src}\n" + "\n".join(lines) + "\n")
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    subprocess.run(cmd, check=True)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", probe_obj, "-o", PROBE_LIB], check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
