"""WP-SGD hot path for AMD MI355X: k sequential SGD chains of unequal length and one
weighted model average (Algorithm 1 of arXiv 1708.04801), as a C-ABI HIP library with a
thin ctypes binding."""
