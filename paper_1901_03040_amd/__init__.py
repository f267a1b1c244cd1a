"""MI355X (gfx950) implementation of the QESGD quantize / aggregate / update hot path.

``binding`` is the ctypes front end of the C-ABI library built from ``csrc/``;
``synth`` draws the seeded synthetic inputs.  Nothing is loaded at import time:
the first call into ``binding`` loads the shared library and raises if it has
not been built.
"""
__all__ = ["binding", "synth"]
