"""MI355X-native MoE layer (forward + backward) behind a C-ABI HIP library.

`paper_2109_10465_amd.binding` is the thin ctypes layer over the library;
`paper_2109_10465_amd.inputs` generates the seeded synthetic workloads.
Importing the package does not load the library; the first call into
`binding` does and fails loudly if it has not been built.
"""
