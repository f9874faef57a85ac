"""MI355X-native HAG aggregation: host search + HIP kernels behind a C ABI.

Submodules:
  binding -- ctypes front end of libhag (argument marshalling only)
  synth   -- seeded synthetic graphs / features (no aggregation arithmetic)
"""
__all__ = ["binding", "synth"]
