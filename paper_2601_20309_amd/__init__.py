"""MI355X-native KV-cache rotation engine (DuplexKV of the SuperInfer paper,
Section 4.3.2): HIP kernels behind a C ABI, plus a thin ctypes binding.

`workloads` (seeded synthetic inputs) imports without the built library;
`binding` needs paper_2601_20309_amd/libduplexkv.so and fails loudly without it.
"""
