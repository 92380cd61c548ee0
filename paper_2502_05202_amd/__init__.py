"""MI355X-native TLI (token-level intersection) draft-and-verify path.

`synth` draws the seeded synthetic workloads; `binding` is the thin ctypes layer over the C-ABI
library built from `csrc/` (it raises if the library is missing -- there is no CPU fallback).
"""
