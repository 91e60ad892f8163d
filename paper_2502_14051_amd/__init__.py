"""MI355X-native RocketKV hot path (hybrid sparse attention over a SnapKV-compressed cache).

The compute lives in ``csrc/`` (HIP kernels for gfx950 behind a C ABI declared
in ``include/rocketkv.h``); ``rocketkv`` is the thin ctypes binding and
``workloads`` draws seeded synthetic inputs.  Importing this package does not
load the native library; the binding loads it on first use and raises if it
has not been built.
"""
__all__ = ["rocketkv", "workloads"]
