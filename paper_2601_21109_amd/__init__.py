"""ChunkWise LoRA hot path for AMD MI355X (gfx950): hand-written HIP kernels behind a C ABI
(``include/cwl.h``) with a thin ctypes binding (``binding``).  ``workloads`` holds the seeded
synthetic input generators.  The HIP library is loaded on first use and its absence is an
error: there is no CPU fallback."""
__all__ = ["binding", "workloads", "build"]
