"""libtbn: MI355X-native inference kernels for tiled-bit layers (Tiled Bit Networks).

Importing the package is cheap; the HIP library is loaded on first use of
``paper_2407_12075_amd.tbn``.
"""
