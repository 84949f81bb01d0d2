"""Builds libfoldconv.so in-tree with hipcc for gfx950.

Usage: ``python -m paper_2601_11608_amd.build`` (or ``build()`` from Python).
"""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfoldconv.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

COMMON = ["-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function", "-fvisibility=hidden"]
# Packed-fp32 VALU forms are disabled for all device code.
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# Per-file device flags.  The dense-walk kernel keeps 216 registers of filter fragments per lane; it pins them
# to the AGPR half of the register file and asks the compiler to put the MFMA results in VGPRs, where the
# epilogue's VALU instructions read them directly (otherwise every finished tile costs 64 v_accvgpr_read).
PER_FILE = {"conv_stream_lds.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def device_flags(src):
    return DEVICE + PER_FILE.get(os.path.basename(src), [])


def build(verbose=False):
    """Compile every source under csrc/ and link the shared library."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))
    procs = []
    objs = []
    for s in srcs:
        o = os.path.join(objdir, os.path.basename(s) + ".o")
        objs.append(o)
        cmd = [HIPCC] + COMMON + (device_flags(s) if s.endswith(".hip") else ["-x", "c++"]) + ["-c", s, "-o", o]
        if s.endswith(".cpp"):
            cmd = ["g++"] + COMMON + ["-c", s, "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for s, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            print("FAILED: %s\n%s" % (s, out), file=sys.stderr)
        elif out.strip() and verbose:
            print(out)
    if failed:
        raise RuntimeError("libfoldconv build failed")
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
