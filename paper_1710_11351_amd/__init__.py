"""MI355X-native gradient aggregation + update step (ChainerMN's Allreduce +
optimize steps, Section 2.3 of the paper) — HIP kernels behind a C-ABI library
with a thin ctypes binding.  Importing the package does not load the library;
`paper_1710_11351_amd.binding` does, and fails loudly if it was not built."""
