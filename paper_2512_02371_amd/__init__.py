"""Five image-processing stages as dense products on the MI355X matrix units.

The compute lives in the C-ABI library built from ``csrc/`` (declared in
``include/hb.h``); :mod:`paper_2512_02371_amd.hb` is a thin ctypes binding and
:mod:`paper_2512_02371_amd.synth` draws the seeded benchmark inputs.
Nothing is loaded at import time; ``hb.load()`` raises if the library is missing.
"""
__all__ = ["hb", "synth"]
