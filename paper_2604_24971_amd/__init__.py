"""PolyKV shared-pool hot path for MI355X (gfx950): HIP kernels behind a C-ABI library
(`csrc/`, declared in `include/polykv.h`) and a thin ctypes binding (`polykv`)."""
