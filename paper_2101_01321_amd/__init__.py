"""libibert: integer-only encoder layer (I-BERT) for AMD MI355X (gfx950).

``synth`` (seeded synthetic inputs) imports nothing heavy.  ``binding`` loads the HIP shared
library on first use and fails loudly when it has not been built.
"""
__all__ = ["synth", "binding"]
