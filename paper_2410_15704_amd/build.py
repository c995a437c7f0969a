"""Build librvq.so (the C-ABI library) in-tree with hipcc for gfx950.

    python -m paper_2410_15704_amd.build [--force]
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librvq.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 VALU forms are switched off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(ROOT, "include", "rvq.h")]
    return any(os.path.getmtime(p) > t for p in deps)


# Per-file extra flags.  The screen kernel reduces matrix-core results with min3 / med3 chains;
# without -fno-honor-nans every operand would first be re-quieted by an extra VALU instruction.
EXTRA = {"rvq_encode_screen.hip": ["-fno-honor-nans"]}


def build(force: bool = False, verbose: bool = True) -> str:
    """Compile every csrc/*.hip to an object under csrc/_build/ and link librvq.so."""
    if not force and not stale():
        return LIB
    bdir = os.path.join(CSRC, "_build")
    os.makedirs(bdir, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    hdr_t = max(os.path.getmtime(p) for p in
                glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(ROOT, "include", "rvq.h")])
    objs, procs = [], []
    for src in sources():
        name = os.path.basename(src)
        obj = os.path.join(bdir, name.replace(".hip", ".o"))
        objs.append(obj)
        if (not force and os.path.exists(obj)
                and os.path.getmtime(obj) > max(os.path.getmtime(src), hdr_t)):
            continue
        cmd = ["hipcc", *FLAGS, *EXTRA.get(name, []), *os.environ.get("RVQ_EXTRA_FLAGS", "").split(),
               *inc, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stderr=subprocess.PIPE, text=True)))
    for cmd, pr in procs:
        _, err = pr.communicate()
        err = "\n".join(l for l in err.splitlines() if "packed-fp32-ops" not in l)
        if err.strip():
            print(err, file=sys.stderr)
        if pr.returncode:
            raise subprocess.CalledProcessError(pr.returncode, cmd)
    link = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
