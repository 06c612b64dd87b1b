"""MoQAE inference hot path for AMD MI355X (gfx950): chunk routing, mixed-precision
quantize-and-pack, and decode attention over the packed KV cache.

`binding` is the ctypes front-end of the C-ABI library (include/moqae.h);
`synth` draws the seeded synthetic workloads; `build` compiles the library.
"""
