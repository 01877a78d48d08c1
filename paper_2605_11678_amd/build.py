"""Compile the native parts in-tree: the HIP library (hipcc, gfx950), and the
plain-C input generator (gcc).  Nothing here runs on the GPU."""
import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB_PATH = os.path.join(PKG, "libdemand_layering.so")
SYNTH_PATH = os.path.join(PKG, "synth", "libsynth.so")

HIP_SOURCES = [
    "dl_api.hip",
    "dl_host.cpp",
    "kernels_gemm.hip",
    "kernels_attn.hip",
    "kernels_misc.hip",
    "kernels_decode.hip",
]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-fno-gpu-rdc",
]


def _run(cmd, quiet_pat=None):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = p.stdout
    if quiet_pat:
        out = "\n".join(l for l in out.splitlines() if quiet_pat not in l)
    if p.returncode != 0:
        sys.stderr.write(out + "\n")
        raise RuntimeError("command failed: " + " ".join(cmd))
    if out.strip():
        sys.stderr.write(out + "\n")


def hipcc_path():
    for c in ("/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if c and os.path.exists(c):
            return c
    raise RuntimeError("hipcc not found")


def build_synth():
    src = os.path.join(PKG, "synth", "synth.c")
    _run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", SYNTH_PATH, src, "-lm"])
    return SYNTH_PATH


def build_lib(jobs=8):
    """hipcc every source to an object (in parallel), then link one shared library."""
    hipcc = hipcc_path()
    bdir = os.path.join(PKG, "_build")
    os.makedirs(bdir, exist_ok=True)
    procs = []
    objs = []
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    for s in HIP_SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(bdir, os.path.splitext(s)[0] + ".o")
        objs.append(obj)
        lang = ["-x", "hip"] if s.endswith(".hip") else []
        cmd = [hipcc] + HIPCC_FLAGS + inc + lang + ["-c", src, "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs)
    _drain(procs)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objs,
         quiet_pat="packed-fp32-ops")
    return LIB_PATH


def _drain(procs):
    err = None
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            sys.stderr.write(out + "\n")
            err = RuntimeError("command failed: " + " ".join(cmd))
        elif out.strip():
            sys.stderr.write(out + "\n")
    procs.clear()
    if err:
        raise err


def build_all():
    build_synth()
    build_lib()


def ensure_built():
    """Build only what is missing (tests, smoke and bench load what is there)."""
    if not os.path.exists(SYNTH_PATH):
        build_synth()
    if not os.path.exists(LIB_PATH):
        build_lib()


if __name__ == "__main__":
    build_all()
    print(LIB_PATH)
