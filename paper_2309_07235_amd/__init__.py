"""MI355X-native LU (no pivoting), Cholesky and 3mm kernels behind a C ABI.

``paper_2309_07235_amd.binding`` wraps the shared library built from ``csrc/``;
``paper_2309_07235_amd.inputs`` holds the seeded synthetic input generators.
Nothing is imported eagerly so that the input generators stay usable on a
machine without the HIP runtime.
"""
__all__ = ["binding", "inputs", "build"]
