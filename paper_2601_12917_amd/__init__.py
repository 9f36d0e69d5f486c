"""MI355X-native client-side ZGR step (hand-written HIP kernels behind a C ABI).

`binding` mirrors include/zgr.h; `session` owns the torch device memory that
the library works on; `build` compiles the kernels for gfx950.
"""
