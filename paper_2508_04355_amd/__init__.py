"""Grid-code protected GEMM for MI355X (gfx950): Python binding over the C-ABI library."""
