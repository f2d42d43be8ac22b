"""MI355X-native sensitivity pass of QuantuneV2 (arXiv 2501.07161): HIP kernels
behind a C ABI (`libqv2.so`), a ctypes binding of the same names, and seeded
synthetic inputs.  `binding` loads the native library on first use and raises
if it has not been built; there is no CPU fallback."""
