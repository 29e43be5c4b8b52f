"""MI355X-native Dictionary Annealing (arXiv 1509.05194, Sec. 3.1): the heat / cool /
re-encode sweep over M additive dictionaries, as HIP kernels for gfx950 behind a C ABI.

`hclae`  -- ctypes binding of libhclae.so (argument marshalling only)
`synth`  -- seeded synthetic inputs shaped like the paper's workloads
"""
__all__ = ["hclae", "synth"]
