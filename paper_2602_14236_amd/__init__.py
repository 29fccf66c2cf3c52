"""MI355X-native Sali-Cache pre-attention filter (HIP library `libsali` + ctypes binding).

`binding` loads the library on first use and raises if it has not been built;
`synth` draws the seeded benchmark inputs and can be imported without a GPU.
"""
__all__ = ["binding", "synth", "build"]
