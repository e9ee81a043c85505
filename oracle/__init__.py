"""CPU oracle for the draft-tree hot path of Recursive Speculative Decoding.

TEST INFRASTRUCTURE ONLY.  Everything under this package is a plain, slow,
fp64 NumPy implementation written from the paper's equations and algorithms.
It shares no code with the HIP path and must never be imported by the product
package; only the test-suite, the smoke check and the CPU-baseline leg of the
benchmark call it.

Modules
-------
philox          counter-based Philox4x32-10 generator, uniform and Gumbel maps
gumbel_topk     Gumbel-Top-k sampling without replacement (RSD-C sampler)
sbs             one Stochastic Beam Search step (RSD-S sampler)
tree_attention  dense tree-masked attention in fp64
rrs             recursive rejection sampling (single level and over a tree)
filter_kv       FilterKVCache: the accepted path's rows appended to the cache
prob_filter     top-k / nucleus (top-p) filtering of a logit row

Every function is pinned by tests/test_oracle_*.py to something other than
itself (known-answer vectors, exact enumeration, closed forms, library
routines); no function here is "parity unpinned".
"""
