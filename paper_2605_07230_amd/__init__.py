"""MI355X-native tree-verification step of CASCADE speculative image decoding.

``binding`` loads the HIP library (``libcascade_verify.so``, built in-tree by
``__graft_entry__.build()``) and exposes the four C entry points under the same
names; it raises if the library is missing — there is no CPU fallback.
``workloads`` draws the seeded synthetic inputs.
"""
