"""Bit-reproducible synthetic node features, roughly N(0, 1).

Element (v, k) of a table with `dim` columns is a pure function of
(seed, v * dim + k): one 64-bit word is split into four 16-bit integers whose
sum (an Irwin-Hall variate, mean 131070, variance 4 * (2**32 - 1) / 12) is
centred in integer arithmetic and scaled by one fp32 multiply. The integer to
fp32 conversion is exact (|x| < 2**24) and the multiply is a single IEEE
operation, so a host and a device implementation of this recipe produce the
same bits; that is what lets a CPU checker regenerate the few rows it needs of
a table that only exists in device (or pinned host) memory.

fp16 tables hold the same values rounded to nearest-even.
"""
import numpy as np

from . import rng

# 1 / sqrt(4 * (2**32 - 1) / 12) rounded to fp32; the device fill kernel uses the same bits
SCALE_BITS = 0x37DDB3D7
SCALE = np.array([SCALE_BITS], dtype=np.uint32).view(np.float32)[0]
CENTRE = 131070  # 4 * 65535 / 2
_MASK16 = np.uint64(0xFFFF)


def feature_key(seed):
    return rng.make_key(seed, 0xFEA7)


def feature_rows(seed, node_ids, dim, dtype=np.float32):
    """Rows of the synthetic feature table for the given node ids: [len(ids), dim]."""
    ids = np.asarray(node_ids, dtype=np.int64).astype(np.uint64)
    key = feature_key(seed)
    out = np.empty((ids.shape[0], dim), dtype=dtype)
    cols = np.arange(dim, dtype=np.uint64)
    step = max(1, (1 << 22) // max(dim, 1))
    for lo in range(0, ids.shape[0], step):
        ctr = ids[lo:lo + step, None] * np.uint64(dim) + cols[None, :]
        w = rng.u64(key, ctr)
        s = (w & _MASK16) + ((w >> np.uint64(16)) & _MASK16) + ((w >> np.uint64(32)) & _MASK16) + (w >> np.uint64(48))
        x = (s.astype(np.int64) - CENTRE).astype(np.float32) * SCALE
        out[lo:lo + step] = x.astype(dtype)
    return out
