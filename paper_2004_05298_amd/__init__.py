"""DEF / DEF-A compression-and-update step (arXiv 2004.05298) for MI355X.

`binding` is the ctypes front end of the HIP library; `workloads` holds the
seeded input generators; `build` compiles the library with hipcc.
"""
