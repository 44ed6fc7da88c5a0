"""MI355X-native request load predictor + load anticipator (PreServe, Sec. 3.3 / 3.4.1).

``workloads`` holds the seeded input generators; ``binding`` is the thin ctypes layer over
the C-ABI library built from ``csrc/``.  Importing this package loads nothing native."""
