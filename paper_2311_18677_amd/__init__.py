"""MI355X-native decode attention (the token-generation step's hot path).

`binding` wraps the C ABI of include/sw_decode.h (libsw_decode.so, hand-written
HIP for gfx950); `workloads` holds the seeded synthetic batch generators.
Importing the package does not load the library; calling into it does, and
fails loudly if it has not been built.
"""
__version__ = "0.1.0"
