"""Builds libtreekv.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtreekv.so")
SOURCES = ["treekv_host.hip", "treekv_decode.hip", "treekv_prefill.hip", "treekv_prompt.hip", "treekv_wavelet.hip",
           "treekv_probe.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]
# The prefill kernels take maxima of MFMA results, which never hold NaNs; telling the compiler so saves the
# instruction per operand that would quiet signalling NaNs and lets it fuse pairs of maxima into v_max3_f32.
PER_FILE_FLAGS = {"treekv_prefill.hip": ["-fno-honor-nans"]}


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every source for gfx950 and link the shared library.  Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    noise = "is not a recognized feature for this target"   # the host pass does not know the packed-fp32 feature
    objdir = tempfile.mkdtemp(prefix="treekv_build_")
    try:
        jobs = []
        for src in SOURCES:
            obj = os.path.join(objdir, src + ".o")
            cmd = [hipcc, *FLAGS, *PER_FILE_FLAGS.get(src, []), *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            jobs.append((obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        logs, failed = [], False
        for obj, proc in jobs:
            out, _ = proc.communicate()
            logs.append("\n".join(l for l in out.splitlines() if noise not in l))
            failed |= proc.returncode != 0
        if not failed:
            tmp = LIB + f".{os.getpid()}.tmp"
            cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *[o for o, _ in jobs]]
            if verbose:
                print(" ".join(cmd), flush=True)
            res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            logs.append(res.stdout)
            failed = res.returncode != 0
            if failed and os.path.exists(tmp):
                os.remove(tmp)
        log = "\n".join(l for l in logs if l.strip())
        if failed:
            raise RuntimeError("hipcc failed:\n" + log)
        if verbose and log.strip():
            print(log)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(objdir, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
