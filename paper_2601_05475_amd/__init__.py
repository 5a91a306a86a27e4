"""MI355X-native shared-prefix candidate decoding and scoring (MaxCode search hot path).

``synth`` holds the seeded input recipes; ``binding`` is the ctypes layer over the
C-ABI library built from ``csrc/``.  Importing the package loads neither."""
