"""MI355X-native integer-only CNN inference: Python binding of the C boundary
declared in include/icnn.h.  PyTorch supplies device memory and streams only;
every operation runs in the library's HIP kernels.  There is no CPU fallback:
if the compiled library is missing, importing `binding` raises.
"""
