"""PSO-PS synchronization step on one MI355X: hand-written HIP kernels behind
a C-ABI library, with a thin ctypes binding."""
