"""MI355X-native TORQ hot path: two-level rotation + MXFP4 quantisation + W4A4 GEMM.

`synth` (input generators) imports nothing from the HIP side; `binding` loads
the C-ABI library and fails loudly when it is missing.
"""
