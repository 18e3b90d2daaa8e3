"""MI355X-native cached denoising step of dLLM-Cache (arXiv 2506.06295).

`binding` wraps the C ABI of libdllmc.so (hand-written gfx950 HIP kernels);
`inputs` holds the seeded synthetic workloads.  Importing the package loads
nothing; the library is opened on first use and its absence is an error.
"""
