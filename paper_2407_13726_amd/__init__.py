"""MI355X-native packed structured tensor contractions (DASTAC hot path).

``paper_2407_13726_amd.dastac`` is the thin ctypes binding over the C-ABI
library ``libdastac_hip.so`` (HIP kernels for gfx950); ``inputs`` holds the
seeded synthetic input streams.  Nothing here falls back to a CPU path: the
binding raises if the library has not been built.
"""
