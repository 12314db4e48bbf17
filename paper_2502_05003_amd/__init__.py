"""QuEST quantized-linear hot path for AMD MI355X (gfx950): HIP kernels behind a C ABI.

`paper_2502_05003_amd.binding` exposes the C-ABI entry points on torch device tensors;
`paper_2502_05003_amd.synth` draws the seeded synthetic workloads.  Nothing is imported
eagerly so that the input generators can be used without the HIP library.
"""
