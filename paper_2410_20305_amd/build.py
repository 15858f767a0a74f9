"""Compile libpsattn.so for gfx950 with hipcc (in-tree, next to this file)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpsattn.so")
LAYER_LIB = os.path.join(HERE, "libpsattn_layer.so")   # the attention-layer benchmark: libpsattn + rocBLAS
SOURCES = ["psattn_meta.cpp", "psattn_pack.cpp", "psattn_api.hip", "psattn_generic.hip", "psattn_mfma_fwd.hip", "psattn_mfma_bwd.hip",
           "psattn_mfma_dkdv.hip", "psattn_bwd_static.hip", "psattn_probe.hip", "psattn_rope.hip", "psattn_logprob.hip"]

# Packed-fp32 VALU instructions are switched off for all device code (the compiler
# otherwise forms them from ordinary float arithmetic).
DEVICE_FLAGS = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

# The dK/dV kernel manages the accumulation registers a[0:191] itself (see the head of its
# source file); the compiler must not park spilled values there.
SOURCE_FLAGS = {"psattn_mfma_dkdv.hip": ["-mllvm", "-amdgpu-spill-vgpr-to-agpr=0"],
                # the forward takes its row maxima with fmaxf; without NaNs to honour that is one v_max3_f32 per
                # three values (the kernels require finite inputs)
                "psattn_mfma_fwd.hip": ["-fno-honor-nans"],
                # the probe measures the hardware fp32 atomic add, not a compare-and-swap loop
                "psattn_probe.hip": ["-munsafe-fp-atomics"]}

def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def device_asm(src: str, out: str) -> str:
    """Compiles one source of csrc/ to gfx950 assembly with the library's own flags (for
    checks on register use); returns the text."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-x", "hip", "-I", os.path.join(ROOT, "include"),
           "-I", CSRC, *DEVICE_FLAGS, *SOURCE_FLAGS.get(src, []), "-S", "--cuda-device-only", "-w",
           os.path.join(CSRC, src), "-o", out]
    subprocess.check_call(cmd)
    with open(out) as f:
        return f.read()


def build(verbose: bool = True, extra=()) -> str:
    """Always recompiles; returns the path of the shared library."""
    objs = []
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(bdir, src + ".o")
        cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC, *DEVICE_FLAGS, *SOURCE_FLAGS.get(src, []), *extra,
               "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(ln for ln in out.splitlines() if "packed-fp32-ops" not in ln)
        if out.strip() and verbose:
            print(out)
        if p.returncode != 0:
            failed = True
            print("compile failed: %s" % src, file=sys.stderr)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    # the layer library: host code only, links libpsattn.so (found next to it at run time) and rocBLAS
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip",
           "-I", os.path.join(ROOT, "include"), os.path.join(CSRC, "psattn_layer.cpp"), "-o", LAYER_LIB,
           "-L", HERE, "-lpsattn", "-L/opt/rocm/lib", "-lrocblas", "-Wl,-rpath,$ORIGIN", "-Wl,-rpath,/opt/rocm/lib"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build()
