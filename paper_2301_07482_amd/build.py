"""Build libfreshgnn.so (HIP, gfx950) in-tree with hipcc. `python -m paper_2301_07482_amd.build`.

Every source is compiled to an object of its own (in parallel), then linked. With FG_BUILD_INCREMENTAL=1 in the
environment a source whose object is newer than it and than every header is not compiled again; without it
everything is compiled on every call."""
import glob
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libfreshgnn.so")
OBJ_DIR = os.path.join(HERE, "_build")
# -packed-fp32-ops is switched off: scalar and float2 code is left to unpacked fp32 instructions
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def hipcc():
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def build_library(verbose=True):
    srcs = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))
    headers = glob.glob(os.path.join(HERE, "csrc", "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    incremental = os.environ.get("FG_BUILD_INCREMENTAL") == "1"
    os.makedirs(OBJ_DIR, exist_ok=True)
    includes = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            return obj
        cmd = [hipcc()] + HIPCC_FLAGS + includes + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
        objs = list(pool.map(compile_one, srcs))
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc"] + objs + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
