"""KVCrush per-layer KV-cache compression for MI355X (gfx950).

`paper_2503_00022_amd.binding` is the thin ctypes layer over the C-ABI library
built from `csrc/`; `paper_2503_00022_amd.pipeline` holds the two call sequences
over it (a layer after prefill, a cache during decoding) with their buffers;
`paper_2503_00022_amd.inputs` generates the seeded synthetic workloads.  Nothing is imported eagerly so that the workload generator can be
used without the GPU library.
"""
