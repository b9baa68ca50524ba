"""Build the HIP library in-tree: paper_2502_02493_amd/libeasyspec.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libeasyspec.so")
SOURCES = ["easyspec.cpp", "gemv.hip", "attention.hip", "util.hip", "accept.hip"]
HEADERS = [os.path.join(CSRC, "kernels.h"), os.path.join(CSRC, "device_common.hpp"), os.path.join(CSRC, "launch_common.hpp"), os.path.join(CSRC, "tile_index.hpp"),
           os.path.join(HERE, "..", "include", "easyspec.h"), os.path.join(HERE, "..", "include", "easyspec_instrument.h")]

# -packed-fp32-ops off: the compiler must not form packed fp32 VALU instructions.
HIPCC_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    for p in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if p and (os.path.sep not in p or os.path.exists(p)):
            return p
    raise RuntimeError("hipcc not found")


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library.  Returns its path."""
    if not force and not stale():
        return LIB
    objs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc(), *HIPCC_FLAGS, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            sys.stderr.write(r.stdout + r.stderr)
            raise RuntimeError(f"hipcc failed on {src}")
        noise = "is not a recognized feature for this target"
        rest = [l for l in r.stderr.splitlines() if l.strip() and noise not in l]
        if rest and verbose:
            print("\n".join(rest), flush=True)
        objs.append(obj)
    tmp = LIB + f".tmp{os.getpid()}"
    subprocess.check_call([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
