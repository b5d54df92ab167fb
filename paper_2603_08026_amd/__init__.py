"""MI355X (gfx950) library for DyLLM's per-denoising-step sparse layer update.

csrc/     hand-written HIP kernels and the C ABI (include/dyllm.h)
binding   ctypes marshalling onto libdyllm.so
layer     device-memory holder used by tests and the bench
build     hipcc driver
"""
