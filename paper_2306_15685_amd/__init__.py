"""Contextual-biasing WFST beam-search decoder for MI355X (gfx950).

The decoder itself is the HIP library under ``csrc/`` behind a C ABI
(``include/cbd.h``); ``binding`` marshals arguments to it, ``synth`` makes the
seeded synthetic inputs.  Nothing here falls back to a CPU path.
"""
__all__ = ["synth", "binding"]
