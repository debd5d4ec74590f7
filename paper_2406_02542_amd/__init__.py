"""MI355X-native Loki decode attention (arXiv 2406.02542): HIP kernels behind a C ABI.

``paper_2406_02542_amd.api`` is the thin binding over ``libloki.so``;
``paper_2406_02542_amd.synth`` generates the seeded synthetic workloads;
``paper_2406_02542_amd.build`` compiles the library in-tree.
"""
__all__ = ["api", "synth", "build"]
