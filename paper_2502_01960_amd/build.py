"""Build libmpic.so for gfx950 with hipcc (in-tree, next to this file)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmpic.so")
PROBE_LIB = os.path.join(HERE, "libmpic_probe.so")   # measurement aid (bench.py --mfma-ceiling), not part of the product library
PROBE_SOURCES = ["probe_mfma.hip", "probe_read.hip"]
SOURCES = ["plan.cpp", "api.hip", "assemble.hip", "attn_f32.hip", "attn_bf16.hip", "decode.hip", "select.hip", "store.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed fp32 instructions are switched off for device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose=False, extra=()):
    """Compile every translation unit and link the shared library.  Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    procs = []
    # the product library, and every source once more with -DMPIC_PROBE_BUILD (plus the matrix-core
    # probe) for the probe library: the same code with the timing-only kernel variants compiled in
    for probe in (False, True):
        for src in SOURCES + (PROBE_SOURCES if probe else []):
            obj = os.path.join(obj_dir, src + (".probe.o" if probe else ".o"))
            cmd = [hipcc, *FLAGS, *extra, *(["-DMPIC_PROBE_BUILD"] if probe else []), "-x", "hip", "-c",
                   os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            procs.append((probe, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs, probe_objs = [], []
    for src, obj, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {obj}:\n{out}")
        if verbose and out.strip():
            print(out)
        (probe_objs if src else objs).append(obj)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], check=True)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *probe_objs, "-o", PROBE_LIB], check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
