"""CPU oracle for the ARCQuant hot path (arXiv 2601.07475).

TEST INFRASTRUCTURE ONLY.  This package is the plain, slow, obviously-correct
statement of what the GPU library computes.  It may be imported by the tests,
by the smoke check and by the benchmark's CPU-baseline leg, and by nothing
else; the product path never routes through it.  It shares no code with the
HIP kernels and imports nothing from the GPU package.

Modules
-------
formats    E2M1 element grid and E4M3 block-scale byte: decode tables and
           round-to-nearest-even encoders written as "nearest table entry,
           ties to the even code" (Appendix A, Table "formats").
arcquant   the method: per-block NVFP4 quantization (Section 3.1 eq. (1)),
           the online activation quantizer with augmented residual channels
           (Section 3.2 steps (1)-(3)), the offline weight packer
           (Section 3.2 "Offline Weight Quantization"), dequantization and
           the fp64 product over the extended reduction dimension
           (Section 3.2 eq. (2)).
brute      a second, deliberately different implementation (exact rationals,
           explicit loops) used only to pin the first on tiny inputs.

Parity status: every function here is pinned by tests/test_oracle_*.py
against format definitions, closed forms, invariants, the paper's error
bounds, a library fp8 cast and brute force.  The paper prints no worked
numeric example, so the exact output bytes for realistic inputs are fixed by
the documented readings of the paper, not by a printed value.
"""
