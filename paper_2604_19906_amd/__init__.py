"""MI355X-native batched inverse-Helmholtz tensor-product operator.

``paper_2604_19906_amd.tpo``        thin ctypes binding over the C-ABI library (libtpo.so)
``paper_2604_19906_amd.workloads``  seeded synthetic inputs (no operator arithmetic)
``paper_2604_19906_amd.build``      compiles the HIP sources for gfx950 into libtpo.so

Importing the package loads nothing; the binding loads the library on first use and raises
if it has not been built.
"""

__all__ = ["tpo", "workloads", "build"]
