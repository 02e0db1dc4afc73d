"""K-FAC preconditioner step for CNN layers on MI355X (gfx950).

``paper_2007_00784_amd.kfac`` is the thin ctypes binding over the C-ABI HIP
library (``csrc/``, declared in ``include/kfac.h``); ``synthetic`` holds the
seeded workload generators.  Importing the package does not load the native
library; the binding does, and raises if it has not been built.
"""
