"""MI355X-native matrix-free dense MTTKRP (hot path of arxiv 2510.14891).

``paper_2510_14891_amd.binding`` is the thin ctypes layer over the C-ABI
library built from ``csrc/``; ``paper_2510_14891_amd.inputs`` makes seeded
synthetic workloads.  Importing the package itself loads nothing, so the input
generators stay usable on a machine where the HIP library has not been built;
every compute entry point raises if the library is missing.
"""
__all__ = ["binding", "inputs", "build"]
