"""MI355X-native MoE-layer hot path of an expert-aware multi-batch pipeline.

``binding``  ctypes front end of the C-ABI library built from ``csrc/`` (hand-written HIP)
``build``    in-tree hipcc build for gfx950
``inputs``   seeded synthetic workloads (shared with the tests' CPU oracle)
"""
