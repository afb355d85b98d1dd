"""2:4 semi-structured-sparse conv2d for AMD MI355X (gfx950): Python binding over the C-ABI library."""
