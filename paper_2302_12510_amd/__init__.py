"""DyBit quantize + GEMM/conv hot path for AMD MI355X (gfx950).

`binding` holds the ctypes front end of libdybit.so (the HIP library), `synth` the seeded
synthetic workloads, `build` the in-tree hipcc build.  Nothing here computes on the CPU.
"""
