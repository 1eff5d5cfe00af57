"""Consensus draft construction across parallel sampling paths on MI355X.

`synth` draws the seeded synthetic inputs; `binding` is the thin ctypes layer
over the C-ABI library built from `csrc/` (imported lazily so that the input
generators stay usable where the HIP library has not been built).
"""
