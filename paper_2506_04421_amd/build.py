"""Builds libhmar_attn.so (HIP kernels + C ABI) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libhmar_attn.so")

SOURCES = ["api.cpp", "schedule.cpp", "fwd.hip", "bwd.hip", "no_alloc.hip"]

# -packed-fp32-ops off: hipcc must not form v_pk_*_f32 from the fp32 softmax arithmetic.
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def variant_path(name: str) -> str:
    """Where a measurement variant of the library is written (never the library the package loads)."""
    return os.path.join(HERE, f"libhmar_attn_{name}.so")


def build_library(verbose: bool = False, variant: str = "", defines=()) -> str:
    """Compile every source and link the shared library.  Always recompiles.
    With `variant`, builds libhmar_attn_<variant>.so with the given -D knobs (see the list at the
    top of csrc/device_common.h) next to the library instead: for measurements only."""
    out = variant_path(variant) if variant else LIB_PATH
    cmd = [hipcc_path(), "-O3", "-std=c++17", "-fPIC", "-shared", "-x", "hip", *DEVICE_FLAGS,
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, *[f"-D{d}" for d in defines],
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", out + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError(f"hipcc failed building {os.path.basename(out)}")
    os.replace(out + ".tmp", out)
    return out


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--variant", default="", help="build libhmar_attn_<variant>.so for measurements")
    ap.add_argument("-D", dest="defines", action="append", default=[], help="macro for the variant, e.g. -DHMAR_TUNE_LDS_PAD_FWD=32768")
    a = ap.parse_args()
    if a.defines and not a.variant:
        ap.error("-D knobs need --variant: the library the package loads is always built without them")
    print(build_library(verbose=True, variant=a.variant, defines=a.defines))
