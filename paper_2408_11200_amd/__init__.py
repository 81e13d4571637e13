"""MI355X-native local B-spline KAN / UKAN layer (forward and backward).

The compute lives in the HIP library built from `csrc/` (C ABI declared in
`include/kan.h`); `binding` is the thin ctypes front end with the same entry
point names.  Importing this package does not load the library; the first call
into `binding` does, and fails loudly when it has not been built.
"""
__all__ = ["binding", "autograd", "workloads", "roofline"]
