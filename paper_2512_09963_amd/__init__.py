"""MI355X-native verification step of GoodSpeed's central verification server.

`synth` holds the seeded input generators; `binding` is the thin ctypes layer
over the C-ABI library built from `csrc/` (imported on demand: it needs torch
and the built shared object).
"""
