"""MI355X-native GEMM over micro-structured unified / pruned weights (arXiv 2106.08301).

`paper_2106_08301_amd.binding` is the Python face of the C-ABI library (include/muw.h) and needs the
built HIP library; `paper_2106_08301_amd.synth` (seeded inputs, workload shapes) needs numpy only.
"""
