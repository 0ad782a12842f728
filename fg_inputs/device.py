"""Feature tables filled where they live (HBM or pinned host memory) by a small HIP kernel that
implements the recipe of `features.py` bit for bit. Input generation only."""
import ctypes as C
import glob
import os
import shutil
import subprocess

import numpy as np

from . import features

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfg_inputs.so")


def build_library(verbose=True):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + \
        sorted(glob.glob(os.path.join(_HERE, "csrc", "*.hip"))) + ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_PATH


_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run fg_inputs.device.build_library()")
        _lib = C.CDLL(LIB_PATH)
        _lib.fgin_fill_features.restype = C.c_int
        _lib.fgin_fill_features.argtypes = [C.c_void_p, C.c_uint64, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_void_p]
    return _lib


def feature_table(seed, num_nodes, dim, dtype="f32", location="hbm"):
    """A [num_nodes, dim] torch tensor of synthetic features in HBM, or in pinned host memory (location="host")."""
    import torch
    td = torch.float32 if dtype == "f32" else torch.float16
    if location == "host":
        t = torch.empty((num_nodes, dim), dtype=td, pin_memory=True)
    else:
        t = torch.empty((num_nodes, dim), dtype=td, device="cuda")
    key = int(features.feature_key(seed))
    rc = _load().fgin_fill_features(t.data_ptr(), key, 0, num_nodes, dim, t.element_size(),
                                    torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError(f"fgin_fill_features failed with {rc}")
    torch.cuda.synchronize()
    return t
