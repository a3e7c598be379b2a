"""MI355X-native Dynamic-aware Operator (Long Exposure, Sec. VI).

Sub-modules:
  inputs -- seeded synthetic workload generators (no method arithmetic).
  lx     -- thin ctypes binding of the C-ABI HIP library (fails loudly if the
            library has not been built).

Nothing is imported eagerly so that the input generators can be used on a
machine without the HIP library.
"""
