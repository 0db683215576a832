"""MI355X-native linear-relaxation bound propagation for transformer verification.

The product is the C-ABI library `lib/libtv.so` (sources in `csrc/`, API in `include/tv.h`);
`binding` is its thin ctypes wrapper.  Importing this package does not load the library.
"""
__all__ = ["binding"]
