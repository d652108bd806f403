"""MI355X-native NOVAK update step: HIP kernels behind a C ABI (libnovak.so) and its ctypes binding.

`paper_2601_07876_amd.novak` holds the binding (same names as include/novak.h);
`paper_2601_07876_amd.build` compiles the library in-tree with hipcc for gfx950.
"""
