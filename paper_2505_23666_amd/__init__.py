"""MI355X-native LoLA attention layer (arxiv 2505.23666): HIP kernels behind a C ABI.

``paper_2505_23666_amd.binding`` holds the thin ctypes front end (same names as ``include/lola.h``);
importing this package loads nothing.
"""
