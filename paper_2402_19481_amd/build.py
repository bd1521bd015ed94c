"""Builds libdistrifusion.so (gfx950) in-tree with hipcc: one object per source, then one link."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdistrifusion.so")
SOURCES = ["api.hip", "refresh.hip", "groupnorm.hip", "conv_gemm.hip", "wgemm.hip", "attn.hip", "elementwise.hip", "unet.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# The tuning build (python -m paper_2402_19481_amd.build --tuning) compiles the environment switches in (DF_TILE,
# DF_SPLITK, DF_ATTN_SPLITS, ...: kernel-selection overrides for sweeps such as `bench.py --tile-sweep`) and writes
# libdistrifusion_tune.so beside the library; the library proper never reads the environment.
OBJ_TUNE = os.path.join(HERE, "_build_tune")
LIB_TUNE = os.path.join(HERE, "libdistrifusion_tune.so")


def _compile(src, tuning=False):
    obj = os.path.join(OBJ_TUNE if tuning else OBJ, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, *(["-DDF_TUNING"] if tuning else []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose=True, tuning=False):
    os.makedirs(OBJ_TUNE if tuning else OBJ, exist_ok=True)
    srcs = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(lambda s: _compile(s, tuning), srcs))
    lib = LIB_TUNE if tuning else LIB
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build(tuning="--tuning" in sys.argv)
