"""SEA attention forward pass for MI355X (gfx950): thin Python binding over the C-ABI HIP library."""
