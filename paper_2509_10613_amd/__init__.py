"""MI355X-native batched signature kernels (Goursat-PDE solve, forward and exact backward).

The HIP library is loaded lazily by :mod:`paper_2509_10613_amd.binding`; importing the package itself
needs neither a GPU nor the built library (``workloads`` is plain numpy).
"""
