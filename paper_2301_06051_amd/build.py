"""Builds libdsvt.so (HIP, gfx950 only) in-tree with hipcc."""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdsvt.so")
OBJ_DIR = os.path.join(PKG, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=fast",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function"]


PHASE_LIB = os.path.join(OBJ_DIR, "libdsvt_phase.so")    # the layer kernel with its optional phase clocks (csrc/phase_clock.h)


def _compile(src, extra=(), suffix=".o"):
    obj = os.path.join(OBJ_DIR, os.path.basename(src) + suffix)
    r = subprocess.run([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj], capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        print(err)
    return obj


def build_library(verbose=True):
    """Compile every csrc/*.hip for gfx950 and link libdsvt.so next to this file."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    if not srcs:
        raise RuntimeError("no HIP sources found")
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources")
    return LIB


def build_phase_library(verbose=True):
    """The same library with -DDSVT_PHASE_CLOCKS on layer.hip, beside the product library's objects (which must have
    been built): what `python -m paper_2301_06051_amd.phase_clocks` loads.  Nothing else loads it."""
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    objs = [os.path.join(OBJ_DIR, os.path.basename(src) + ".o") for src in srcs if os.path.basename(src) != "layer.hip"]
    missing = [o for o in objs if not os.path.exists(o)]
    if missing:
        raise RuntimeError(f"build the product library first ({missing[0]} is missing)")
    objs.append(_compile(os.path.join(CSRC, "layer.hip"), ("-DDSVT_PHASE_CLOCKS",), ".phase.o"))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PHASE_LIB, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {PHASE_LIB}")
    return PHASE_LIB


if __name__ == "__main__":
    build_library()
    build_phase_library()
