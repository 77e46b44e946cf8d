"""MI355X-native offloaded sparse decoding (KVDrive hot path): HIP kernels behind
a C-ABI library plus a thin ctypes binding.  Importing the package does not load
the library; `paper_2605_18071_amd.kvd` does, and fails loudly if it is not built."""
