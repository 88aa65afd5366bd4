"""CSR5 SpMV for AMD MI355X: HIP library (csrc/, include/csr5.h) plus a thin
ctypes binding.  `workloads` holds the seeded input generators.  Nothing is
loaded at import time; `binding.load()` opens libcsr5.so on first use."""
