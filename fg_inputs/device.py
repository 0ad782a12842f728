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
        _g = [C.c_int64, C.c_uint64, C.c_uint64, C.c_uint64] + [C.c_double] * 6 + [C.c_uint64, C.c_uint64]
        _lib.fgin_chunglu_degrees.restype = C.c_int
        _lib.fgin_chunglu_degrees.argtypes = _g + [C.c_void_p, C.c_void_p]
        _lib.fgin_chunglu_indices.restype = C.c_int
        _lib.fgin_chunglu_indices.argtypes = _g + [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        _lib.fgin_grad_norms.restype = C.c_int
        _lib.fgin_grad_norms.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_uint64, C.c_void_p, C.c_void_p]
    return _lib


def grad_norms(ids, n_dev_ptr, max_n, key, out, stream):
    """out[i] = the synthetic gradient norm of node ids[i] under `key` (see workload.grad_norms) for i below the
    device-side count at address n_dev_ptr (None: max_n), on `stream` (a raw stream handle)."""
    rc = _load().fgin_grad_norms(ids.data_ptr(), n_dev_ptr, max_n, int(key), out.data_ptr(), stream)
    if rc != 0:
        raise RuntimeError(f"fgin_grad_norms failed with {rc}")


def chunglu_csr(graph):
    """The Chung-Lu graph `graph` written out as an in-neighbour CSR in HBM: (indptr int64 [N + 1], indices int32 [E]).
    Evaluated on the device, so single entries can differ from `graph.neighbour` on the host (another pow); the CSR
    returned is the graph for whoever samples from it."""
    import torch
    g = graph
    args = [g.num_nodes, g._a, g._ainv, g._b, float(g.c), float(g.r0), float(g.alpha), float(g._lo), float(g._span),
            1.0 / float(g._e), int(g._key_deg), int(g._key_nbr)]
    st = torch.cuda.current_stream().cuda_stream
    deg = torch.empty(g.num_nodes, dtype=torch.int64, device="cuda")
    rc = _load().fgin_chunglu_degrees(*args, deg.data_ptr(), st)
    if rc != 0:
        raise RuntimeError(f"fgin_chunglu_degrees failed with {rc}")
    indptr = torch.zeros(g.num_nodes + 1, dtype=torch.int64, device="cuda")
    torch.cumsum(deg, 0, out=indptr[1:])
    del deg
    edges = int(indptr[-1].item())
    indices = torch.empty(max(edges, 1), dtype=torch.int32, device="cuda")
    rc = _lib.fgin_chunglu_indices(*args, indptr.data_ptr(), edges, indices.data_ptr(), st)
    if rc != 0:
        raise RuntimeError(f"fgin_chunglu_indices failed with {rc}")
    torch.cuda.synchronize()
    return indptr, indices[:edges]


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
