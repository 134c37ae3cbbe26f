"""MI355X-native hot path of Bidirectional Sparse Attention: HIP kernels behind a C ABI
(include/bsa.h, built into libbsa.so) and a thin ctypes binding (binding.py)."""
