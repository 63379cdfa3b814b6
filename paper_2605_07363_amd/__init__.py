"""MI355X-native MISA indexer (block-pool, route heads, score tokens, top-k, re-rank).

``paper_2605_07363_amd.misa`` is the ctypes binding of the HIP library and
raises at import if the library has not been built; ``workloads`` only draws
synthetic inputs and needs no GPU.
"""
