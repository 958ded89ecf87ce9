"""APMSqueeze compression-stage hot path for MI355X (gfx950): Python side.

`binding` wraps the C-ABI library `libapms.so` (hand-written HIP kernels);
`workloads` generates the seeded synthetic inputs.  Importing this package
does not load the library; `binding` does, and fails loudly when it is absent.
"""
