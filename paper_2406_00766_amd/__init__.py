"""MI355X-native forward / backward passes of compiled probabilistic circuits.

`workloads` holds the seeded input generators; `binding` is the thin ctypes layer over the
C-ABI library built from `csrc/` (loaded lazily, so importing this package never needs a GPU).
"""
