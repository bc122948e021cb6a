"""MI355X-native mini-batch HGNN layer path (merged features, merged CSR, one launch per stage).

`binding` holds the ctypes mirror of include/hgnn.h, `runner` the call order for a whole
mini-batch, `build` the hipcc build of libhgnn.so.  Importing `binding` or `runner` fails
loudly when the shared library has not been built.
"""
