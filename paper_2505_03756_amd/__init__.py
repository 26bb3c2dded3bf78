"""MI355X-native paged multi-LoRA layer step over a unified caching pool.

`paper_2505_03756_amd.flpool` is the thin ctypes binding of the C-ABI library
(`include/flpool.h`); `paper_2505_03756_amd.workload` draws seeded synthetic
inputs.  Nothing here computes: every step of the path runs in the HIP kernels
under `csrc/`.
"""
