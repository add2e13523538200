"""MI355X-native stage-level partition search (RaNNC, Sec. III-C): HIP kernels behind a
C ABI, plus a thin ctypes binding.  Importing the package does not load the library;
`paper_2103_16063_amd.binding` does, and fails loudly if it has not been built."""
