"""Builds libintfa.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(_HERE), "include")
LIB = os.path.join(_HERE, "libintfa.so")
SOURCES = ["intfa_attention.hip", "intfa_attention_fewq.hip", "intfa_attention_half.hip", "intfa_quantize.hip"]

# Packed-fp32 instructions are switched off on purpose (the flag is a device-side feature; the host
# pass warns that it does not know it, which is harmless).  No fast-math: the quantizer is bit-exact.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-ffp-contract=off", "-Wall", "-Wno-unused-command-line-argument"]


def build(verbose: bool = False, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-I", INCLUDE, "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(ln for ln in res.stdout.splitlines() if "packed-fp32-ops" not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


MICROBENCH_SRC = os.path.join(CSRC, "microbench", "issue_model.hip")
MICROBENCH_BIN = os.path.join(_HERE, "issue_model_microbench.bin")


def build_microbench(verbose: bool = False) -> str:
    """The stand-alone issue-model micro-benchmark (register-only probes of the MFMA / vector ALU / exp pipes)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument", MICROBENCH_SRC, "-o", MICROBENCH_BIN]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(ln for ln in res.stdout.splitlines() if "packed-fp32-ops" not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return MICROBENCH_BIN


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_microbench(verbose=True))
