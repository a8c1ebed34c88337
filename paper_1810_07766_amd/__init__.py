"""MI355X-native lossy partitioned model averaging (RPS, arXiv 1810.07766).

`paper_1810_07766_amd.rps` binds the C ABI declared in include/rps.h; importing it
requires the built HIP library (python -m paper_1810_07766_amd.build).
"""
