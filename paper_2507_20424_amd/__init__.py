"""DPPF consensus-round kernels for MI355X (gfx950): Python binding over the C-ABI library.

Importing the package does not load the native library; the first call into
``paper_2507_20424_amd.dppf`` does, and raises if it has not been built."""
