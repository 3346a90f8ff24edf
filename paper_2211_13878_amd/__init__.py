"""MI355X-native batched plan-search dynamic program (paper section 3.3, Eq. 1).

`workloads` draws the seeded synthetic inputs; `binding` is the thin ctypes
layer over the C-ABI HIP library (libgalvdp.so).  Importing the package does
not load the library; the binding does so on first use and fails loudly when
it has not been built.
"""
from . import workloads  # noqa: F401
