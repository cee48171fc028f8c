"""MI355X-native ShadowSync hot path: HIP kernels behind a C-ABI library, a thin ctypes
binding (`binding`), and seeded synthetic workloads (`synth`).  Importing the package
loads nothing; `binding.load()` opens the built library and fails loudly if it is
missing."""
