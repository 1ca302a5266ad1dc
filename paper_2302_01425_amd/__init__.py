"""MI355X-native (gfx950, hand-written HIP) p-norm-regularised top-k mask / top-k-in-magnitude.

``paper_2302_01425_amd.binding`` is the thin ctypes layer over the C-ABI library built from
``csrc/``; it raises if the library is missing (there is no CPU fallback).  ``workloads`` holds the
seeded input generators only.
"""
