"""MI355X-native quantized GEMM (u8 x s8 -> u8) with fused offsets and requantization.

`paper_2101_05615_amd.qgemm`     thin ctypes binding of the C-ABI library (needs the built HIP library)
`paper_2101_05615_amd.workloads` seeded synthetic inputs (numpy only)

Nothing is imported eagerly so that the input generators stay usable on a machine
without a GPU; importing `qgemm` fails loudly when the HIP library is not built.
"""
__all__ = ["qgemm", "workloads"]
