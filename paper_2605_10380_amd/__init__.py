"""MI355X-native extend / verify path (paged KV, greedy draft verification).

The package holds the HIP sources (``csrc/``), the ctypes binding over the C ABI
(``binding``) and the seeded synthetic-input generators (``inputs``).  Nothing is
imported eagerly: ``inputs`` is pure numpy and is shared with the CPU oracle's tests,
``binding`` loads the compiled library and fails loudly when it is missing.
"""

__all__ = ["inputs", "binding"]
