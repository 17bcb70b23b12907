"""BPDQ per-layer quantization pass for MI355X (gfx950): Python binding of the C-ABI
library `libbpdq.so` plus the seeded synthetic workloads.  The compute lives entirely
in the HIP library; importing this package does not load it (see `binding`)."""
