"""MI355X-native Hadamard Binary Matrix Multiply (HBMM).

``paper_1905_10759_amd.hbmm`` is the thin binding over the C-ABI library built from
``csrc/``; ``paper_1905_10759_amd.synth`` draws the seeded synthetic workloads.  Nothing is
imported eagerly so that the input generator can be used without the HIP library.
"""
__all__ = ["hbmm", "synth"]
