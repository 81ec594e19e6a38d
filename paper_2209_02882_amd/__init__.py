"""MI355X-native CSR SpMM with segment-group reductions (gfx950 HIP kernels
behind a C-ABI library).  Importing the package loads nothing native; the
binding loads the shared library on first use and raises if it is absent."""

__version__ = "0.1.0"
