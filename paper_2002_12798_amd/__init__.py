"""amap: composed access maps for chains of layout operators, executed by
single gfx950 kernels.  See include/amap.h for the C ABI; `binding` wraps it
one to one, `device` holds the PyTorch glue (device memory and streams only)."""
