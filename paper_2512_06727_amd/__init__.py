"""MI355X-native KV-CAR decode hot path: ctypes binding over libkvcar.so.

`paper_2512_06727_amd.binding` is the thin Python layer over the C ABI declared
in include/kvcar.h; `paper_2512_06727_amd.synth` holds the seeded synthetic
workloads.  Nothing is loaded at import time: the shared library is opened on
first use and its absence is an error, never a fallback.
"""
__all__ = ["binding", "synth", "build"]
