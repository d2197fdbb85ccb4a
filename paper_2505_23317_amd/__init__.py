"""MI355X-native coarse-to-fine detection-transformer encoder (CF-DETR A1-A3).

``paper_2505_23317_amd.cfdetr`` is the ctypes binding over the C-ABI library
built from ``csrc/``; ``paper_2505_23317_amd.synth`` draws seeded synthetic
workloads.  Nothing is loaded at package import time.
"""
