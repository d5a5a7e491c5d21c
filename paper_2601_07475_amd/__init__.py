"""ARCQuant hot path for AMD MI355X (gfx950): fused NVFP4 activation quantizer with
augmented residual channels, offline weight packer and the W4A4 GEMM over K' = K + S.

`binding` wraps the C-ABI library libarcq.so (hand-written HIP); `workloads` makes the
seeded synthetic inputs; `build` compiles the library.  Importing this package loads
nothing native; `binding.lib()` does, and raises if the library has not been built.
"""
__version__ = "0.1.0"
