"""pshard: MI355X-native hot path of pipelined sharding (planner + streamed layer-stack forward).

The package is a thin ctypes binding over libpshard.so (see include/pshard.h).  Nothing here
computes: every step of the path runs in the HIP library.  Import `binding` to load it.
"""
