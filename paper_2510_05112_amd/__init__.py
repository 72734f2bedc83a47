"""fpsched: MI355X-native batched evaluation of candidate pipeline schedules.

Thin ctypes binding over ``libfpsched.so`` (HIP, gfx950).  It only marshals
arguments: every step of the hot path -- dependency propagation, per-candidate
reductions, top-k -- runs in the library's kernels.  PyTorch provides device
memory and the stream, nothing else.  There is no CPU fallback: if the library
is missing or no GPU is present, the device calls raise.
"""
from .binding import (FLAG_DEADLOCK, FLAG_INCOMPLETE, FLAG_OVER_CAP, FpschedError, Problem,
                      library_path, load_library, version)

__all__ = ["Problem", "FpschedError", "load_library", "library_path", "version",
           "FLAG_DEADLOCK", "FLAG_INCOMPLETE", "FLAG_OVER_CAP"]
