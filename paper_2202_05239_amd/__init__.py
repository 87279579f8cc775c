"""MI355X-native 8-bit fixed-point inference kernels (the F8Net layer arithmetic).

`workloads` draws the seeded synthetic operands; `binding` is the thin ctypes layer
over the C-ABI library built from `csrc/` (argument marshalling only).
"""
