"""MI355X-native draft-tree hot path of Recursive Speculative Decoding.

The compute lives in the HIP library `librsd.so` behind the C ABI declared in
include/rsd.h; `binding` marshals torch device tensors into it.  Nothing here
falls back to a CPU implementation: calling an op without the built library or
without a GPU raises.
"""
__all__ = ["binding", "workloads", "draft_tree", "build"]
