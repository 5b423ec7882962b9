"""MI355X-native sparse hot path of Distributed Equivalent Substitution (DES) training.

Sub-modules
-----------
``des``    thin ctypes binding over the C-ABI library ``libdes.so`` (HIP kernels for gfx950).
``synth``  seeded synthetic recommender-shaped batches (no DES arithmetic lives there).

Nothing is imported eagerly: ``synth`` is usable without the HIP library, and ``des`` raises
a clear error as soon as it is imported when the library has not been built.
"""

__all__ = ["des", "synth"]
