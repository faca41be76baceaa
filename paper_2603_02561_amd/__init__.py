"""SVD-Attention for MI355X (gfx950): thin Python binding over the C-ABI library.

`paper_2603_02561_amd.synth` (numpy only) builds the seeded synthetic workloads;
everything else needs `libsolar.so`, built in-tree by `paper_2603_02561_amd.build`.
The binding is loaded lazily so that the input generators import without a GPU.
"""

__all__ = ["binding", "synth", "build"]
