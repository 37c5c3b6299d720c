"""MI355X-native hot path of Progressive Stochastic Binarization (arxiv 1904.02205).

`psb` is the thin binding over the C-ABI library (include/psb.h); `synth` draws
the synthetic workloads.  Importing the package does not load the HIP library.
"""
__all__ = ["psb", "synth"]
