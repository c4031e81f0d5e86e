"""MI355X-native EDEN (arXiv 2108.08842) encode / decode / mean.

`paper_2108_08842_amd.eden` is a thin ctypes binding over the C-ABI library built from `csrc/`
(`libeden_hip.so`, hand-written HIP kernels for gfx950).  `paper_2108_08842_amd.synth` holds the seeded
synthetic input generators used by the tests and the benchmark.  Importing the package loads nothing;
the library is loaded on first use and a missing library is an error, never a fallback.
"""
