"""MI355X-native hot path of PAROAttention (arXiv 2506.16054): token reorder, block-wise
quantization and block-sparse INT8 attention as hand-written gfx950 HIP kernels behind a
C-ABI shared library.  ``paper_2506_16054_amd.binding`` is the thin ctypes layer over it;
``paper_2506_16054_amd.workloads`` generates the seeded synthetic inputs."""
