"""MI355X-native RainFusion2.0 block-sparse attention layer (HIP kernels behind a C ABI).

`paper_2512_24086_amd.rf2` is the thin ctypes binding of librf2.so;
`paper_2512_24086_amd.inputs` holds the synthetic workload generator;
`paper_2512_24086_amd.build` compiles the library for gfx950.
Nothing is imported eagerly so that the input generator can be used without the library.
"""
__version__ = "0.1.0"
