"""Inverted Activations (arXiv 2407.15545) for AMD MI355X: HIP kernels behind a C ABI.

`paper_2407_15545_amd.binding` is the thin ctypes layer over libinvact.so;
`paper_2407_15545_amd.nn` holds the PyTorch layers built on it;
`paper_2407_15545_amd.build` compiles the library.
"""
