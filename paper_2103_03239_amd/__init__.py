"""Moshpit All-Reduce group-averaging rounds on one MI355X (gfx950).

``paper_2103_03239_amd.binding`` is the thin ctypes layer over the C-ABI
library ``libmoshpit.so`` (hand-written HIP kernels); ``inputs`` holds the
seeded synthetic workloads.  Importing the package loads nothing native.
"""
