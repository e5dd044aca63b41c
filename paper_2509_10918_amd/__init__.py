"""ToMA (Token Merge with Attention) layer path for AMD MI355X: select -> merge -> attention -> unmerge.

The compute lives in the HIP library under csrc/ (C ABI declared in include/toma.h); `binding`
marshals torch device tensors into it.  Nothing here falls back to the CPU.
"""
