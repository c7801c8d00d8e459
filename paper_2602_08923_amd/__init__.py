"""MI355X-native hot path of DynamiQ's compressed multi-hop all-reduce.

The kernels live in csrc/ behind the C ABI declared in include/dq.h; binding.py
is the thin ctypes layer with the same names.  Nothing here falls back to a CPU
implementation: calling into the path without the built library raises.
"""
