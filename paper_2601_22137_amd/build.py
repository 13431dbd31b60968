"""Builds libprism.so (HIP, gfx950) in-tree with hipcc.  Run as `python -m paper_2601_22137_amd.build`."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libprism.so")
BUILD_DIR = os.path.join(HERE, "_build")

SOURCES = ["prism_api.hip", "gemm_f32.hip", "gemm_bf16.hip", "chain.hip", "dbnewton.hip", "fit.hip", "misc.hip", "sketch.hip"]
COMMON = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-I" + os.path.join(ROOT, "include"),
          "-I" + CSRC, "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
# the sketch generator is specified as unfused IEEE operations
PER_FILE = {"sketch.hip": ["-ffp-contract=off"]}


def build(verbose=True):
    """Compiles every source and links libprism.so.  PRISM_EXTRA_HIPCC_FLAGS (build-time environment
    variable, empty by default) appends compiler flags, e.g. -DPRISM_AB_SWITCHES for a development
    build whose kernel choices can be switched through the environment."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    extra = os.environ.get("PRISM_EXTRA_HIPCC_FLAGS", "").split()
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(BUILD_DIR, src.replace(".hip", ".o"))
        cmd = [hipcc] + COMMON + extra + PER_FILE.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and verbose:
            print(out, flush=True)
        if p.returncode != 0:
            failed = True
            print("FAILED: " + src, file=sys.stderr)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return OUT


if __name__ == "__main__":
    build()
