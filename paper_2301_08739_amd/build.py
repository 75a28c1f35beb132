"""Compile libflatformer.so for gfx950 with hipcc (in-tree, next to this file)."""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libflatformer.so")
PEAKS_LIB = os.path.join(HERE, "libffpeaks.so")   # bench-only: stream copy and MFMA issue loop (csrc/bench/peaks.hip)

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instruction selection is switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))


# Per-file flags (both builds of the fused layer kernel get the same set).  It takes maxima of matrix-core results; without the promise
# that no NaN is involved every such maximum costs an extra canonicalising instruction.
EXTRA_FLAGS = {"layer_mfma.hip": ["-fno-honor-nans"], "layer_mfma_f16.hip": ["-fno-honor-nans"]}


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    common = [f for f in HIPCC_FLAGS if f != "-shared"] + ["-I" + os.path.join(ROOT, "include")]
    objs = []
    procs = []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        objs.append(obj)
        cmd = [hipcc] + common + EXTRA_FLAGS.get(os.path.basename(src), []) + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)))
    for cmd, pr in procs:
        _, stderr = pr.communicate()
        err = "\n".join(l for l in stderr.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + err)
        if verbose and err.strip():
            print(err, file=sys.stderr)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB + ".tmp"], verbose)
    os.replace(LIB + ".tmp", LIB)
    _run([hipcc] + HIPCC_FLAGS + [os.path.join(HERE, "csrc", "bench", "peaks.hip"), "-o", PEAKS_LIB + ".tmp"], verbose)
    os.replace(PEAKS_LIB + ".tmp", PEAKS_LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
