"""MUXQ quantized linear layer for MI355X (gfx950): HIP kernels behind a C ABI.

`binding` holds the ctypes front end of libmuxq.so; `synth` the seeded input
generators; `build` compiles the library.  Importing the package loads nothing
heavy; the shared library is opened on first use and its absence is an error.
"""
