"""MI355X (gfx950) implementation of one tensor-parallel rank's fused sliced GEMM +
ring reduce-scatter reduction + track & trigger path of T3 (arXiv 2401.16677).

`binding` is the ctypes front end of the C ABI in include/t3.h (libt3.so, built by
`build`); `workloads` draws the seeded synthetic inputs.
"""
