"""MI355X-native conv2d forward / backward-data / backward-weight.

`paper_1512_01274_amd.mxc` is the binding over the C-ABI library (HIP kernels for
gfx950); `paper_1512_01274_amd.inputs` holds the benchmark layer shapes and the
seeded input generators.  Importing the package itself loads nothing native.
"""
__all__ = ["inputs", "mxc"]
