"""CollectiveKV decode hot path for AMD MI355X (gfx950).

`paper_2601_19178_amd.ckv` is the thin ctypes binding of the C-ABI library (libckv.so);
`paper_2601_19178_amd.workloads` holds the seeded input generators.  Importing the package
itself loads neither the GPU library nor torch; `ckv` loads both (torch first).
"""
