"""MuKV hot path for MI355X (gfx950): HIP kernels behind a C ABI.

`binding` wraps the shared library built from `csrc/` (it raises if the library
is missing -- there is no CPU fallback); `synth` draws the seeded synthetic
streams used by tests and the benchmark.  Nothing is loaded at import time.
"""
