"""Compression step of Compressed PagedAttention for MI355X (gfx950).

``paper_2603_08743_amd.binding`` is the thin ctypes layer over the C-ABI library
``libzp.so`` (hand-written HIP kernels); ``paper_2603_08743_amd.workloads`` makes
seeded synthetic inputs.  Nothing here computes on the CPU: without the built
library and a GPU every call fails loudly.
"""
