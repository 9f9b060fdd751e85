"""MI355X-native CO3 gradient codec (arXiv 2204.08211): HIP kernels behind the C ABI of
include/co3.h, with a ctypes binding of the same names.  Import `binding` to use it."""
