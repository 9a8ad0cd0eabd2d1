"""MI355X-native HGF linear layer (Hybrid Gated Flow): HIP kernels behind a C ABI.

`binding` holds the ctypes face of libhgf.so, `synth` the seeded input generators,
`build` compiles the library for gfx950."""
