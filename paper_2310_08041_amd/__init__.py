"""MI355X-native reassembled low-bit linear layer (QLLM, arXiv 2310.08041).

`binding` wraps the C-ABI library libqllm.so (HIP kernels for gfx950); `workloads` draws the seeded
synthetic inputs.  Nothing here falls back to a CPU implementation: without the built library the
binding refuses to import.
"""
