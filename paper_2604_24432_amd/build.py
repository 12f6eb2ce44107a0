"""Build libksa.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libksa.so")
PROBE_LIB = os.path.join(HERE, "libksa_probe.so")   # bench.py's measurement probes (csrc/ksa_probe.hip), not the product
SOURCES = ["ksa_layout.cpp", "ksa_api.cpp", "ksa_prefill.hip", "ksa_prefill_bwd.hip", "ksa_decode.hip", "ksa_cache.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 VALU instructions are kept out of the generated code (hand-written none either)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]
# MFMA results and accumulator inputs in VGPRs: the forward prefill kernel post-processes them with VALU code.  The
# backward kernels hold more accumulators than there are VGPRs and leave the choice to the compiler.
PER_SOURCE = {"ksa_prefill.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}
OBJ_DIR = os.path.join(HERE, "_build")


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the device-only target feature; that warning is expected
    out = "\n".join(ln for ln in res.stdout.splitlines() if "packed-fp32-ops" not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return out


def build(verbose: bool = False, extra=()) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs, procs = [], []
    for s in SOURCES:
        obj = os.path.join(OBJ_DIR, os.path.splitext(s)[0] + ".o")
        objs.append(obj)
        cmd = [HIPCC, *FLAGS, *PER_SOURCE.get(s, []), *extra, "-x", "hip", "-c", os.path.join(CSRC, s), "-o", obj]
        procs.append(subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
    log = []
    failed = False
    for s, pr in zip(SOURCES, procs):
        text = pr.communicate()[0]
        text = "\n".join(ln for ln in text.splitlines() if "packed-fp32-ops" not in ln)
        log.append(text)
        failed |= pr.returncode != 0
    out = "\n".join(t for t in log if t.strip())
    if failed:
        raise RuntimeError("hipcc failed:\n" + out)
    out += _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB])
    out += _run([HIPCC, *FLAGS, *extra, "-shared", "-x", "hip", os.path.join(CSRC, "ksa_probe.hip"), "-o", PROBE_LIB])
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
