"""MI355X-native fused Flash Decode (split-KV partial pass + LSE combine in one kernel).

``paper_2511_02168_amd.binding`` is the ctypes layer over the C-ABI library
(``include/fd.h``); ``paper_2511_02168_amd.inputs`` holds the seeded synthetic
workloads.  Importing the package loads nothing; the library is loaded on the
first call into ``binding`` and a missing build is an error, never a fallback.
"""
__all__ = ["binding", "inputs", "build"]
