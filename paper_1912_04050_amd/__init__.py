"""MI355X-native (min,+) curve algebra for real-time-calculus analysis.

Sub-modules:
  rtc        thin ctypes binding of the C-ABI library (librtc.so, HIP kernels for gfx950)
  workloads  seeded synthetic curve generators (inputs only, no operator arithmetic)
  _build     hipcc driver that compiles csrc/ into librtc.so

Nothing is imported eagerly: ``workloads`` is usable on a machine without the built
library, while ``rtc`` raises at import time when librtc.so is missing.
"""
__all__ = ["rtc", "workloads"]
