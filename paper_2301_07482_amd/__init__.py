"""MI355X-native hot path of mini-batch GNN training with a selective historical-embedding cache.

`binding` exposes the C ABI of libfreshgnn.so one to one (importing it raises if the library has not been
built: there is no fallback); `pipeline` strings the calls together into one training iteration's data
path on torch device buffers; `build` compiles the library with hipcc.
"""
