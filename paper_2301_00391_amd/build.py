"""Builds libpipad.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2301_00391_amd.build [-v] [-D NAME[=VALUE] ...] [-o PATH]

-D passes a macro to every source: the measurement builds the profiles are taken with, e.g.
-D PIPAD_PARTS_MASK=1 (only the class parts of the hub rows run: results incomplete),
-D PIPAD_AGG_DEPTH=8, -D PIPAD_NO_ROW_ORDER.  -o writes the library somewhere else than in-tree;
the binding loads the file the environment variable PIPAD_LIBRARY names instead of the in-tree one.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpipad.so")
SOURCES = ["pipad_api.hip", "pipad_build.hip", "pipad_aggregate.hip", "pipad_transpose.hip",
           "pipad_ceilings.hip"]


def hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: libpipad needs the ROCm toolchain")


def check_private_memory(remarks: str, limit: int = 64) -> None:
    """Fails the build when a kernel keeps more than a few spilled registers in private (scratch)
    memory.  The aggregation kernels take their arguments as one large struct; if the compiler
    cannot prove that it is only read at constant offsets it copies the whole struct (over 2 KB)
    into every lane's private memory, which costs an order of magnitude in run time and no test
    would notice."""
    name = None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif "ScratchSize [bytes/lane]:" in line and name:
            size = int(line.split("ScratchSize [bytes/lane]:")[1].split()[0])
            if size > limit and "5pipad" in name:  # this library's kernels (namespace pipad)
                raise RuntimeError(f"kernel {name} uses {size} bytes of private memory per lane "
                                   f"(limit {limit}): kernel arguments copied to scratch?")


def build(verbose: bool = False, defines=(), output: str = LIB) -> str:
    """Compiles every HIP source for gfx950 and links the shared library.  Always rebuilds."""
    flags = [*[f"-D{d}" for d in defines],
        "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
        # packed fp32 instructions are kept off on this target
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function",
    ]
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", f".{os.getpid()}.o"))
        cmd = [hipcc(), *flags, "-Rpass-analysis=kernel-resource-usage", "-c",
               os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stderr=subprocess.PIPE, text=True)))
        objs.append(obj)
    for cmd, p in procs:
        _, err = p.communicate()
        if p.returncode != 0:
            sys.stderr.write(err)
            raise RuntimeError("hipcc failed: " + " ".join(cmd))
        check_private_memory(err)
    link = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", output, *objs]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    for o in objs:
        os.remove(o)
    return output


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("-v", action="store_true", help="print the compiler command lines")
    ap.add_argument("-D", action="append", default=[], metavar="NAME[=VALUE]")
    ap.add_argument("-o", default=LIB, metavar="PATH")
    a = ap.parse_args()
    print(build(verbose=a.v, defines=a.D, output=a.o))
