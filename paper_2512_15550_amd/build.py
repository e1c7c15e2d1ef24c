"""Compile the HIP library for gfx950 with hipcc, in-tree: two translation units (the host side with
the staged and build kernels; the single-launch decode kernel), compiled side by side, then linked."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
SOURCES = ["ctkvr.hip", "fused.hip"]
LIB = os.path.join(HERE, "libctkvr.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    # every fused multiply-add on a path that decides an integer is written as an explicit fmaf
    "-ffp-contract=off",
    # no packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    jobs = []
    for src in SOURCES:
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, "-c", "-o", obj, os.path.join(CSRC, src)]
        if verbose:
            print(" ".join(cmd))
        jobs.append((obj, cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for obj, cmd, proc in jobs:
        out, _ = proc.communicate()
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
        objs.append(obj)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(link))
    proc = subprocess.run(link, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("link failed:\n" + proc.stdout + proc.stderr)
    return LIB


PROBES = ["sync_probe", "latency_probe", "gather_probe", "xcd_probe"]
PROBE_DIR = os.path.join(HERE, "probes")


def build_probes(verbose: bool = False):
    """The stand-alone measurement programs under csrc/probes (launch floor, in-launch barriers, visibility,
    latencies): executables in probes/, not used by the library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(PROBE_DIR, exist_ok=True)
    out = []
    for name in PROBES:
        exe = os.path.join(PROBE_DIR, name)
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-o", exe, os.path.join(CSRC, "probes", name + ".hip")]
        if verbose:
            print(" ".join(cmd))
        proc = subprocess.run(cmd, capture_output=True, text=True)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + proc.stdout + proc.stderr)
        out.append(exe)
    return out


if __name__ == "__main__":
    import sys
    print(build_library(verbose=True))
    if "--probes" in sys.argv:
        print("\n".join(build_probes(verbose=True)))
