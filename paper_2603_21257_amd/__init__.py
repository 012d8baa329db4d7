"""MI355X-native prefix-hit prefill path (paged KV ingest + paged causal GQA prefill attention).

`binding` is the ctypes view of the C ABI in include/calvo.h, `workload` draws the seeded
synthetic inputs, `build` compiles the HIP library in-tree.
"""
