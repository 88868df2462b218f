"""MI355X-native eviction step + decode attention for Neural Garbage Collection.

``binding`` is the ctypes front end of the HIP library (``libngc.so``, built by
``_build``); ``schedule`` holds the host-side integers of the grow-then-evict
cycle; ``synth`` makes seeded synthetic inputs.  Importing the package loads
nothing: the library is opened on first use and its absence is an error.
"""
from . import schedule, synth  # noqa: F401

__all__ = ["binding", "schedule", "synth"]
