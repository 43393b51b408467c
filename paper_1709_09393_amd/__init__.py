"""MI355X-native Slim-DP communication-set path (score, core select, explore, pack, merge, pull).

The compute lives in ``libslimdp.so`` (hand-written HIP for gfx950 behind a C ABI declared in
``include/slimdp.h``); :mod:`paper_1709_09393_amd.binding` is the thin ctypes layer over it and
:mod:`paper_1709_09393_amd.workloads` draws the seeded synthetic inputs.
"""
__all__ = ["workloads"]
