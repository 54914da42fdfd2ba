"""hipEvent timing through the HIP runtime that is already loaded in the process (ctypes)."""
from __future__ import annotations

import ctypes

import numpy as np


class HipEvents:
    """hipEvent timing on the stream the kernels are launched on (via the HIP runtime already loaded)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so.7")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]

    def create(self) -> int:
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError("hipEventCreate failed: %d" % rc)
        return ev.value

    def record(self, ev: int, stream: int) -> None:
        rc = self.hip.hipEventRecord(ev, stream)
        if rc != 0:
            raise RuntimeError("hipEventRecord failed: %d" % rc)

    def empty_bracket_ms(self, stream: int, reps: int = 64) -> float:
        """Median elapsed time of a start/stop pair with nothing in between: what the two marker
        packets themselves add to every bracketed kernel on this stream."""
        pairs = [(self.create(), self.create()) for _ in range(reps)]
        for a, b in pairs:
            self.record(a, stream)
            self.record(b, stream)
        return float(np.median([self.elapsed_ms(a, b) for a, b in pairs]))

    def elapsed_ms(self, start: int, stop: int) -> float:
        self.hip.hipEventSynchronize(stop)
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), start, stop)
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return float(ms.value)
