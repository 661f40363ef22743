"""LASNet coarse-grained sparse bottleneck on MI355X: HIP kernels behind a C ABI (liblasnet.so),
a ctypes binding (`binding`), and the seeded synthetic-input generator (`synth`)."""
