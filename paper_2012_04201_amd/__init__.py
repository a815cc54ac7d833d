"""MI355X-native batched MLP cross-validation evaluator (HIP kernels behind a C-ABI library).

`inputs` holds the seeded synthetic workloads; `binding` is the thin ctypes layer
over libbbo_mlp.so.  Importing the package does not load the GPU library.
"""
