"""MI355X-native f16 GEMM (C = A B + C) -- C-ABI library plus a thin binding.

`workloads` (input generators) imports nothing else from the package; the
binding in `binding` loads the HIP library on first use and raises if it has
not been built.
"""
