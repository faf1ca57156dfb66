"""MI355X-native local data movement and reduction of MCR-DL's collectives.

``paper_2303_08374_amd.mcr`` is the thin binding of the C-ABI library
(``libmcr.so``, built from ``csrc/``); ``paper_2303_08374_amd.inputs`` holds
the seeded synthetic workloads.  Importing the package loads nothing: the
library is opened on first use of the binding and raises if it is not built.
"""
__all__ = ["inputs", "mcr"]
