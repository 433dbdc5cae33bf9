"""ABFT-protected GEMM for neural-network inference on MI355X (gfx950).

The compute path is the C-ABI library built from ``csrc/`` (hand-written HIP);
``binding`` marshals arguments into it.  Importing the package does not load
the library; the first call does, and fails loudly if it was not built.
"""
