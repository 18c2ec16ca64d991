"""GFormer attention forward for MI355X (gfx950): hand-written HIP kernels behind a C ABI.

`binding` loads the shared library lazily; importing this package does not touch the GPU.
"""
__version__ = "0.1.0"
