"""MI355X-native fused GEMM / batched GEMM / implicit-GEMM conv2d (the scheduled matmul tensor
program of the Hidet paper, Sections 2.2, 3.1, 4 and 5).  The compute lives in the HIP library
under ``csrc/``; ``binding`` is a thin ctypes layer over its C ABI."""
