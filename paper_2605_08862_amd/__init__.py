"""MI355X-native speculative-verification decode step (BubbleSpec hot path).

`binding`  ctypes view of the C ABI in include/bubblespec.h (same names, marshalling only)
`runtime`  torch plumbing: device allocations, stream, paged-cache bookkeeping
`workloads` seeded synthetic inputs (shapes of the paper's workloads; no arithmetic of the method)
`build`    compiles csrc/ with hipcc for gfx950

Every step of the path runs in the HIP library; there is no CPU or PyTorch fallback, and loading
fails loudly when the library has not been built.
"""
