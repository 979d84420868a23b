"""MI355X-native hot path of SQAP-VLA (arXiv 2509.09090): token pruning + W4A4 linears.

`binding` wraps the C ABI of libsqap.so (hand-written gfx950 HIP kernels);
`workloads` generates the seeded synthetic inputs; `build` compiles the library.
"""
