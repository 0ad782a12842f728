"""MI355X-native hot path of mini-batch GNN training with a selective historical-embedding cache.

`binding` exposes the C ABI of libfreshgnn.so one to one; `pipeline` strings the calls together into
one training iteration's data path on torch device buffers.
"""
from . import binding  # noqa: F401  (raises if the HIP library has not been built)
