"""Builds libkvflow.so (HIP kernels + C ABI) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libkvflow.so")
SOURCES = ["kv_api.hip", "kv_copy.hip", "kv_decode.hip", "kv_decode_fp8.hip", "kv_append.hip",
           "kv_prefill.hip", "kv_probe.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
    # packed fp32 VALU forms are kept off for the device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # device code only: no operation here has a NaN operand by design (masked scores are -inf, rows
    # that must not count are zeroed or selected away), so maxima need not quiet signalling NaNs first
    "-Xarch_device", "-fno-honor-nans",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source into one shared library and return its path."""
    cmd = [HIPCC, *FLAGS, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB_PATH


def kernel_resources(source: str) -> dict:
    """Compile one HIP source for the device only and return, per kernel, the registers and scratch bytes the
    compiler reports ({mangled name: {"vgprs": n, "scratch": bytes per lane, "spills": n}})."""
    import re
    import tempfile
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [HIPCC, *[f for f in FLAGS if f not in ("-shared", "-fPIC")], "--cuda-device-only", "-c",
               os.path.join(CSRC, source), "-o", os.path.join(tmp, "dev.o"), "-Rpass-analysis=kernel-resource-usage"]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    out, name = {}, None
    for line in res.stdout.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            out[name] = {}
            continue
        for key, pat in (("vgprs", r" VGPRs: (\d+)"), ("scratch", r"ScratchSize \[bytes/lane\]: (\d+)"),
                         ("spills", r"VGPRs Spill: (\d+)")):
            m = re.search(pat, line)
            if m and name is not None:
                out[name][key] = int(m.group(1))
    return out


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
