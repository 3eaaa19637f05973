"""MI355X-native speculative-round hot path (Fast-ARDiff): HIP kernels + C-ABI + thin binding.

`paper_2512_08537_amd.binding` loads the in-tree libfastardiff.so and raises if it is not built;
`paper_2512_08537_amd.build.build()` compiles it with hipcc for gfx950.
"""

__all__ = ["binding", "build"]
