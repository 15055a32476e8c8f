"""MI355X-native AttnCache hot path (search, map reuse, exact attention).

The GPU entry points live in :mod:`paper_2510_25979_amd.binding` (a ctypes
front-end to ``libattncache.so``); :mod:`paper_2510_25979_amd.synth` holds the
seeded input generators.  Nothing is imported eagerly so that the generators
can be used on machines without the built library.
"""
__all__ = ["binding", "synth", "build"]
