"""MI355X-native sparse-sketch gradient codec (S2 Reducer hot path).

`binding` is the ctypes layer over libs2r.so (include/s2r.h), `pipeline` chains
encode x W -> merge -> decode on device buffers, `workloads` holds the seeded
synthetic gradients, `build` compiles the HIP sources.
"""
