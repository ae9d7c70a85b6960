"""kvx: block-free KV-cache transfer between paged pools on AMD MI355X.

`paper_2408_08147_amd.kvx` is the Python binding of the C-ABI library
(include/kvx.h); `paper_2408_08147_amd.workloads` draws synthetic inputs.
Nothing is loaded at package import time.
"""
