"""ctypes binding of libpaac.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; torch is used for device memory and
streams.  There is no CPU fallback: if the library is missing the import of its symbols raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpaac.so")

PAAC_ARCH_NIPS, PAAC_ARCH_NATURE = 0, 1
PAAC_PREC_FP32, PAAC_PREC_BF16 = 0, 1
PAAC_ALG_ACTOR_CRITIC, PAAC_ALG_NSTEP_Q = 0, 1
ERRORS = {0: "PAAC_OK", -1: "PAAC_E_NULL", -2: "PAAC_E_BADCONFIG", -3: "PAAC_E_WORKSPACE",
          -4: "PAAC_E_HIP", -5: "PAAC_E_STATE"}

# every symbol include/paac.h declares
SYMBOLS = ["paac_workspace_bytes", "paac_create", "paac_destroy", "paac_init_params",
           "paac_select_actions", "paac_select_actions_noalloc", "paac_train_step", "paac_param_count", "paac_get_state",
           "paac_set_state", "paac_get_train_outputs", "paac_get_train_activations", "paac_fill_uniforms", "paac_set_graphs", "paac_set_activation_cache", "paac_set_algorithm",
           "paac_set_profiling", "paac_kernel_times", "paac_flops", "paac_last_error"]


class paac_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("arch", "n_e", "t_max", "n_actions", "in_c", "in_h", "in_w", "precision")]


class paac_hparams(C.Structure):
    _fields_ = [(n, C.c_float) for n in
                ("gamma", "beta", "value_coef", "lr", "rms_alpha", "rms_eps", "clip_norm")]


class paac_train_stats(C.Structure):
    _fields_ = [(n, C.c_float) for n in
                ("policy_loss", "entropy", "value_loss", "total_loss", "grad_norm", "clip_scale")] + \
               [("nonfinite", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """Load libpaac.so (build it first with paper_1705_04862_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_1705_04862_amd.build` (no fallback path exists)")
        L = C.CDLL(LIB_PATH)
        vp, i32, u64, sz = C.c_void_p, C.c_int32, C.c_uint64, C.c_size_t
        L.paac_workspace_bytes.argtypes = [C.POINTER(paac_config), C.POINTER(sz)]
        L.paac_create.argtypes = [C.POINTER(paac_config), vp, sz, vp, C.POINTER(vp)]
        L.paac_destroy.argtypes = [vp]
        L.paac_destroy.restype = None
        L.paac_init_params.argtypes = [vp, u64]
        L.paac_select_actions.argtypes = [vp, vp, vp, vp, vp, vp]
        L.paac_select_actions_noalloc.argtypes = [vp, vp, vp, vp, vp, vp]
        L.paac_train_step.argtypes = [vp, vp, vp, vp, vp, C.POINTER(paac_hparams), vp]
        L.paac_param_count.argtypes = [vp]
        L.paac_param_count.restype = sz
        L.paac_get_state.argtypes = [vp, vp, vp, vp]
        L.paac_set_state.argtypes = [vp, vp, vp]
        L.paac_get_train_outputs.argtypes = [vp, vp, vp, vp]
        L.paac_get_train_activations.argtypes = [vp, C.c_int, C.c_int, C.c_int, vp]
        L.paac_fill_uniforms.argtypes = [vp, u64, u64, vp, sz]
        L.paac_set_graphs.argtypes = [vp, C.c_int]
        L.paac_set_activation_cache.argtypes = [vp, C.c_int]
        L.paac_set_algorithm.argtypes = [vp, C.c_int, C.c_float]
        L.paac_set_profiling.argtypes = [vp, C.c_int]
        L.paac_kernel_times.argtypes = [vp, C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_float),
                                        C.POINTER(i32), C.POINTER(i32)]
        L.paac_flops.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.paac_last_error.argtypes = [vp]
        L.paac_last_error.restype = C.c_char_p
        _lib = L
    return _lib


class PaacError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{ERRORS.get(code, code)}: {msg}")
        self.code = code


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Paac:
    """One PAAC context on the current torch device/stream."""

    def __init__(self, arch: int, n_e: int, t_max: int, n_actions: int, precision: int = 0,
                 stream: Optional[torch.cuda.Stream] = None, device: str = "cuda:0"):
        self.L = lib()
        self.cfg = paac_config(arch, n_e, t_max, n_actions, 4, 84, 84, precision)
        self.device = torch.device(device)
        self.n_e, self.t_max, self.n_actions = n_e, t_max, n_actions
        nbytes = C.c_size_t()
        rc = self.L.paac_workspace_bytes(C.byref(self.cfg), C.byref(nbytes))
        if rc:
            raise PaacError(rc, "paac_workspace_bytes rejected the configuration")
        self.workspace = torch.empty(nbytes.value, dtype=torch.uint8, device=self.device)
        self.stream = stream
        handle = C.c_void_p()
        sptr = None if stream is None else stream.cuda_stream
        with torch.cuda.device(self.device):
            rc = self.L.paac_create(C.byref(self.cfg), self.workspace.data_ptr(), nbytes.value, sptr,
                                    C.byref(handle))
        if rc:
            raise PaacError(rc, "paac_create failed")
        self.ctx = handle
        self.stats_dev = torch.zeros(8, dtype=torch.float32, device=self.device)

    def close(self):
        if getattr(self, "ctx", None):
            self.L.paac_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc:
            raise PaacError(rc, (self.L.paac_last_error(self.ctx) or b"").decode())

    # ---- the three calls of the hot path ----
    def init_params(self, seed: int):
        self._check(self.L.paac_init_params(self.ctx, seed))

    def select_actions(self, states: torch.Tensor, uniforms: torch.Tensor, actions: torch.Tensor,
                       values: Optional[torch.Tensor] = None, probs: Optional[torch.Tensor] = None):
        """states uint8 [n_e,4,84,84]; uniforms f32 [n_e]; actions i32 [n_e] (out); optional
        values f32 [n_e], probs f32 [n_e,A] (out).  All contiguous device tensors."""
        assert states.dtype == torch.uint8 and states.is_contiguous() and states.numel() == self.n_e * 28224
        assert uniforms.dtype == torch.float32 and uniforms.numel() == self.n_e and uniforms.is_contiguous()
        assert actions.dtype == torch.int32 and actions.numel() == self.n_e and actions.is_contiguous()
        assert values is None or (values.dtype == torch.float32 and values.numel() == self.n_e)
        assert probs is None or (probs.dtype == torch.float32 and probs.numel() == self.n_e * self.n_actions)
        self._check(self.L.paac_select_actions(self.ctx, _ptr(states), _ptr(uniforms), _ptr(actions),
                                               _ptr(values), _ptr(probs)))

    def select_actions_noalloc(self, states: torch.Tensor, uniforms: torch.Tensor, actions: torch.Tensor,
                               values: Optional[torch.Tensor] = None, probs: Optional[torch.Tensor] = None):
        """select_actions through the entry point that uses the library's static scratch."""
        assert states.dtype == torch.uint8 and states.is_contiguous() and states.numel() == self.n_e * 28224
        assert uniforms.dtype == torch.float32 and uniforms.numel() == self.n_e and uniforms.is_contiguous()
        assert actions.dtype == torch.int32 and actions.numel() == self.n_e and actions.is_contiguous()
        assert values is None or (values.dtype == torch.float32 and values.numel() == self.n_e)
        assert probs is None or (probs.dtype == torch.float32 and probs.numel() == self.n_e * self.n_actions)
        self._check(self.L.paac_select_actions_noalloc(self.ctx, _ptr(states), _ptr(uniforms), _ptr(actions),
                                                       _ptr(values), _ptr(probs)))

    def train_step(self, states: torch.Tensor, actions: torch.Tensor, rewards: torch.Tensor,
                   dones: torch.Tensor, hp, stats: Optional[torch.Tensor] = None):
        """states uint8 [t_max+1,n_e,4,84,84]; actions i32 / rewards f32 / dones u8 [t_max,n_e];
        hp: object with gamma, beta, value_coef, lr, rms_alpha, rms_eps, clip_norm."""
        B = self.n_e * self.t_max
        assert states.dtype == torch.uint8 and states.is_contiguous() and states.numel() == (B + self.n_e) * 28224
        assert actions.dtype == torch.int32 and actions.numel() == B and actions.is_contiguous()
        assert rewards.dtype == torch.float32 and rewards.numel() == B and rewards.is_contiguous()
        assert dones.dtype == torch.uint8 and dones.numel() == B and dones.is_contiguous()
        h = paac_hparams(hp.gamma, hp.beta, hp.value_coef, hp.lr, hp.rms_alpha, hp.rms_eps, hp.clip_norm)
        st = self.stats_dev if stats is None else stats
        self._check(self.L.paac_train_step(self.ctx, _ptr(states), _ptr(actions), _ptr(rewards),
                                           _ptr(dones), C.byref(h), _ptr(st)))

    # ---- state exchange and helpers ----
    def param_count(self) -> int:
        return int(self.L.paac_param_count(self.ctx))

    def get_state(self, want_grads: bool = True):
        P = self.param_count()
        params = np.empty(P, np.float32)
        rms = np.empty(P, np.float32)
        grads = np.empty(P, np.float32) if want_grads else None
        self._check(self.L.paac_get_state(self.ctx, _np_ptr(params), _np_ptr(rms), _np_ptr(grads)))
        return params, rms, grads

    def set_state(self, params: np.ndarray, rms: Optional[np.ndarray] = None):
        params = np.ascontiguousarray(params, np.float32)
        assert params.size == self.param_count()
        rms = None if rms is None else np.ascontiguousarray(rms, np.float32)
        self._check(self.L.paac_set_state(self.ctx, _np_ptr(params), _np_ptr(rms)))

    def get_train_outputs(self):
        Bp = self.n_e * (self.t_max + 1)
        logits = np.empty((Bp, self.n_actions), np.float32)
        values = np.empty(Bp, np.float32)
        returns = np.empty((self.t_max, self.n_e), np.float32)
        self._check(self.L.paac_get_train_outputs(self.ctx, _np_ptr(logits), _np_ptr(values), _np_ptr(returns)))
        return logits, values, returns

    def get_train_activations(self, layer: int, per_row: int, row0: int = 0, rows: Optional[int] = None) -> np.ndarray:
        """Stored post-ReLU output of conv layer `layer` (NCHW per row) or, for layer = number of conv
        layers, of the hidden fc layer, of the last train step's forward pass; per_row = values per row."""
        rows = self.n_e * (self.t_max + 1) - row0 if rows is None else rows
        out = np.empty((rows, per_row), np.float32)
        self._check(self.L.paac_get_train_activations(self.ctx, layer, row0, rows, _np_ptr(out)))
        return out

    def read_stats(self, stats: Optional[torch.Tensor] = None) -> Dict[str, float]:
        st = (self.stats_dev if stats is None else stats).cpu().numpy()
        out = {n: float(st[i]) for i, n in enumerate(
            ("policy_loss", "entropy", "value_loss", "total_loss", "grad_norm", "clip_scale"))}
        out["nonfinite"] = int(st[6:7].view(np.int32)[0])
        return out

    def fill_uniforms(self, seed: int, offset: int, out: torch.Tensor):
        assert out.dtype == torch.float32 and out.is_contiguous()
        self._check(self.L.paac_fill_uniforms(self.ctx, seed, offset, _ptr(out), out.numel()))

    def set_graphs(self, on: bool):
        self._check(self.L.paac_set_graphs(self.ctx, int(on)))

    def set_activation_cache(self, on: bool):
        self._check(self.L.paac_set_activation_cache(self.ctx, int(on)))

    def set_algorithm(self, algorithm: int, epsilon: float = 0.0):
        """0 = actor-critic (default), 1 = n-step Q-learning with epsilon-greedy selection."""
        self._check(self.L.paac_set_algorithm(self.ctx, int(algorithm), float(epsilon)))

    def set_profiling(self, on: bool):
        self._check(self.L.paac_set_profiling(self.ctx, int(on)))

    def kernel_times(self) -> Dict[str, Dict[str, float]]:
        cap = 64
        names = (C.c_char_p * cap)()
        ms = (C.c_float * cap)()
        calls = (C.c_int32 * cap)()
        n = C.c_int32()
        self._check(self.L.paac_kernel_times(self.ctx, cap, names, ms, calls, C.byref(n)))
        return {names[i].decode(): {"ms": float(ms[i]), "calls": int(calls[i])} for i in range(n.value)}

    def flops(self):
        a, b = C.c_double(), C.c_double()
        self._check(self.L.paac_flops(self.ctx, C.byref(a), C.byref(b)))
        return a.value, b.value
