"""FLToP CTC decoding on MI355X: HIP kernels behind a C-ABI, with a thin ctypes binding."""
