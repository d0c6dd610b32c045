"""MI355X-native hot path of ConQuR's online rotation calibration.

`inputs`  — seeded synthetic activation streams (no method arithmetic).
`binding` — thin ctypes layer over the C-ABI library libconqur.so (HIP kernels).
"""
