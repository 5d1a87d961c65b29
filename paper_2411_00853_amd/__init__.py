"""MI355X-native speculative-sampling verify step: hand-written HIP kernels behind a C ABI
(include/spec_verify.h) plus this thin ctypes binding.  PyTorch is used for device memory and
streams only; every step of the path runs in libspecverify.so."""
