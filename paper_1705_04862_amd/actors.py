"""ctypes binding of the host-side worker pool with the synthetic environment (include/paac_actors.h).
Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpaac_actors.so")
SYMBOLS = ["paac_actors_create", "paac_actors_destroy", "paac_actors_reset", "paac_actors_step",
           "paac_actors_last_step_seconds"]
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run paper_1705_04862_amd/build.py")
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.paac_actors_create.argtypes = [C.c_int32, C.c_int32, C.c_uint64, C.c_float, C.c_int32, C.POINTER(vp)]
        L.paac_actors_destroy.argtypes = [vp]
        L.paac_actors_destroy.restype = None
        L.paac_actors_reset.argtypes = [vp, vp]
        L.paac_actors_step.argtypes = [vp, vp, vp, vp, vp]
        L.paac_actors_last_step_seconds.argtypes = [vp]
        L.paac_actors_last_step_seconds.restype = C.c_double
        _lib = L
    return _lib


class Actors:
    """n_e synthetic environments on n_w worker threads.  Buffers are numpy arrays or pinned torch
    tensors viewed as numpy (host memory); nothing is copied here."""

    def __init__(self, n_e: int, n_w: int, seed: int = 0, p_done: float = 0.01, sprites: int = 24):
        self.L = lib()
        self.n_e, self.n_w = n_e, n_w
        h = C.c_void_p()
        rc = self.L.paac_actors_create(n_e, n_w, seed, p_done, sprites, C.byref(h))
        if rc != 0:
            raise ValueError(f"paac_actors_create failed ({rc})")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.L.paac_actors_destroy(self.h)
            self.h = None

    __del__ = close

    @staticmethod
    def _ptr(a: np.ndarray, dtype, n):
        assert a.dtype == dtype and a.flags.c_contiguous and a.size == n, (a.dtype, a.shape)
        return a.ctypes.data_as(C.c_void_p)

    def reset(self, states: np.ndarray):
        rc = self.L.paac_actors_reset(self.h, self._ptr(states, np.uint8, self.n_e * 4 * 84 * 84))
        assert rc == 0, rc

    def step(self, actions: np.ndarray, states: np.ndarray, rewards: np.ndarray, dones: np.ndarray):
        rc = self.L.paac_actors_step(self.h, self._ptr(actions, np.int32, self.n_e),
                                     self._ptr(states, np.uint8, self.n_e * 4 * 84 * 84),
                                     self._ptr(rewards, np.float32, self.n_e), self._ptr(dones, np.uint8, self.n_e))
        assert rc == 0, rc

    def last_step_seconds(self) -> float:
        return float(self.L.paac_actors_last_step_seconds(self.h))
