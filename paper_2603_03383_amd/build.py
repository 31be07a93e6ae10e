"""Builds libmedusa_hip.so (gfx950) in-tree with hipcc.  Used by __graft_entry__.build()."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmedusa_hip.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-result",
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def build_library(verbose: bool = True, jobs: int = 8) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        cmd = [hipcc, *HIPCC_FLAGS, *os.environ.get("MDZ_EXTRA_HIPCC_FLAGS", "").split(), "-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
        if verbose and r.stderr.strip():
            lines = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l]
            if any("warning" in l or "error" in l for l in lines):
                print("\n".join(lines))
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(compile_one, sources()))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


PROBES = os.path.join(HERE, "probes")
# the stamps probe compiles the library's own kernel sources with their per-workgroup time stamps switched on
PROBE_FLAGS = {"stamps_probe.hip": ["-DMDZ_STAMPS", "-I", os.path.join(os.path.dirname(HERE), "include"), "-I", CSRC]}


def build_probes(verbose: bool = True):
    """Stand-alone measurement programs (probes/*.hip -> probes/<name>): the evidence behind two design decisions,
    not part of the library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = []
    for f in sorted(os.listdir(PROBES)):
        if not f.endswith(".hip"):
            continue
        exe = os.path.join(PROBES, f[:-4])
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", *PROBE_FLAGS.get(f, []), os.path.join(PROBES, f), "-o", exe]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {f}:\n{r.stdout}\n{r.stderr}")
        out.append(exe)
        if verbose:
            print(f"built {exe}")
    return out


if __name__ == "__main__":
    build_library()
    build_probes()
