"""4-bit quantised linear layers (W4A16 group-wise weight-only, W4A4 integer
conv-as-GEMM) for AMD MI355X (gfx950), behind a C-ABI library.

`synth` draws the seeded synthetic inputs; `binding` marshals arguments into
`libqail.so`.  Importing the package does not load the native library; the
first call that needs it does, and fails loudly if it is missing.
"""
__all__ = ["synth", "binding"]
