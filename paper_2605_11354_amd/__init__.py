"""MI355X-native Sparse Linear Attention forward (HIP kernels behind a C ABI, see include/sla.h).

`binding` is the thin ctypes layer over libsla.so, `synth` the seeded input generator,
`build` compiles the library with hipcc for gfx950.
"""
