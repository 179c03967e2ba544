"""MI355X-native packed attention for heterogeneous batches (PackInfer hot path).

Sub-modules:
  workloads -- seeded synthetic inputs (no arithmetic of the method)
  binding   -- ctypes binding of the C-ABI library (libpackinfer.so)
  build     -- hipcc build of the library for gfx950
"""
