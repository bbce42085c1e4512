"""MI355X-native decode attention over QuantSpec's hierarchical 4-bit KV cache.

`binding` wraps the C ABI of libquantspec.so (include/quantspec.h); `synth` draws the seeded
synthetic workloads; `build` compiles the library in-tree.  Importing the package loads nothing.
"""
