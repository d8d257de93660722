"""Compile the HIP sources into the C-ABI shared library (gfx950 only)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libadapm.so")
SOURCES = ["adapm_api.hip", "k_elementwise.hip", "k_gemm64.hip", "k_chol.hip", "k_gemm_mfma.hip", "k_proj_mfma.hip", "k_proj_keep.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]


def build(verbose: bool = False, jobs: int = 8) -> str:
    """Always recompiles every source, then links libadapm.so next to this file."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs)
    _drain(procs)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if out.returncode != 0:
        raise RuntimeError("link failed:\n" + out.stdout)
    return LIB


def build_calibration() -> str:
    """The stand-alone bandwidth measurement csrc/hbm_ceiling.hip (no part of the library, not built by build()):
    plain read / write / read-modify-write kernels of known size.  ./hbm_ceiling prints what HBM delivers for the
    access patterns of the fused kernels; the same kernels under rocprofv3 --pmc give the factors that turn
    FETCH_SIZE / WRITE_SIZE into bytes."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    exe = os.path.join(HERE, "hbm_ceiling")
    cmd = [hipcc, *FLAGS, os.path.join(CSRC, "hbm_ceiling.hip"), "-o", exe]
    out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if out.returncode != 0:
        raise RuntimeError("hipcc failed on hbm_ceiling.hip:\n" + out.stdout)
    return exe


def _drain(procs):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        noise = "packed-fp32-ops"
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        rest = "\n".join(l for l in out.splitlines() if l.strip() and noise not in l)
        if rest.strip():
            print(rest, file=sys.stderr)


if __name__ == "__main__":
    print(build_calibration() if "--calibration" in sys.argv else build(verbose=True))
