"""libfcv2 for MI355X: any-bit quantize/pack codec with spike reserving and bit splitting
(FlashCommunication V2, arxiv 2508.03760) as hand-written HIP kernels behind a C ABI.

`paper_2508_03760_amd.fcv2` is the thin ctypes binding of the C-ABI library; `workloads` holds the seeded
synthetic inputs.  Importing this package does not load the GPU library; the first call does, and fails
loudly if it cannot be built or loaded.
"""
__all__ = ["fcv2", "workloads"]
