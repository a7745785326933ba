"""CurDKV post-prefill KV selection for MI355X (gfx950): HIP kernels behind a
C ABI, a thin ctypes binding, and seeded synthetic workloads."""
