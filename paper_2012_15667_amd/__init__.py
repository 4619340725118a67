"""I/O-lower-bound-tiled forward convolution (direct and Winograd) for AMD MI355X (gfx950)."""
