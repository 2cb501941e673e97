"""MI355X-native hot path of SamKV (multi-context KV cache sparsification + local recomputation).

`paper_2508_11661_amd.samkv` is the ctypes binding of the C-ABI library (HIP kernels for gfx950);
`paper_2508_11661_amd.synth` draws the seeded synthetic workloads.  Importing the package loads neither.
"""
__all__ = ["samkv", "synth"]
