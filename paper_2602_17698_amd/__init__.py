"""MI355X-native (gfx950, hand-written HIP) bitwidth-allocation search of ScaleBITS.

`binding` is the thin ctypes layer over the C-ABI library `libscalebits.so`;
`synth` draws the seeded synthetic inputs.  Importing the package loads nothing
native; the binding loads the library on first use and raises if it is missing.
"""
__all__ = ["binding", "synth"]
