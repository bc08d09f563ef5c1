"""MI355X-native LQER W4A8 linear layer (arXiv 2402.02446).

`paper_2402_02446_amd.binding` is the ctypes face of the C-ABI library
(`liblqer.so`, built from csrc/); `paper_2402_02446_amd.synth` holds the
seeded input generators.  Nothing is imported eagerly: the binding loads the
shared library on first use and raises if it is missing.
"""
