"""Column-wise N:M sparse convolution for MI355X (gfx950).

``paper_2507_17301_amd.binding`` is the thin ctypes layer over the C-ABI library
``libnmconv.so`` (built from ``csrc/`` by ``build.py``); ``workloads`` holds the
synthetic layer tables and seeded generators.  Importing the package loads
nothing native; the library is opened on first use and its absence is an error.
"""
__all__ = ["binding", "workloads", "build"]
