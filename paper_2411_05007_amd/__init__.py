"""MI355X-native SVDQuant W4A4 + low-rank linear layer (arXiv 2411.05007, Eq. 5).

``paper_2411_05007_amd.svdq`` is the thin binding over the C-ABI library
``libsvdq.so`` (HIP kernels for gfx950 + host-side offline quantization);
``paper_2411_05007_amd.inputs`` generates the seeded synthetic layers.
Importing this package does not load the native library; the binding does, and
it raises if the library has not been built.
"""
__all__ = ["inputs", "svdq"]
