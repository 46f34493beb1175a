"""ctypes front end of the CPU oracle (oracle/paac_oracle.cpp) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.  It
imports nothing from the HIP package; a network is described by any object with the attributes
in_c, in_h, in_w, conv (tuples of c_out, kernel, stride), fc and n_actions.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "paac_oracle.cpp")
_LIB = os.path.join(_HERE, "libpaac_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (OpenMP over samples, for timing only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-o", _LIB, _SRC]
        subprocess.check_call(cmd)
    return _LIB


class _Net(C.Structure):
    _fields_ = [("in_c", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32),
                ("n_conv", C.c_int32), ("conv_cout", C.c_int32 * 4), ("conv_k", C.c_int32 * 4),
                ("conv_stride", C.c_int32 * 4), ("fc", C.c_int32), ("n_actions", C.c_int32),
                ("bf16", C.c_int32)]


class _HP(C.Structure):
    _fields_ = [(n, C.c_double) for n in
                ("gamma", "beta", "value_coef", "lr", "rms_alpha", "rms_eps", "clip_norm")]


class _Flips(C.Structure):
    _fields_ = [("units", C.c_int64 * 5), ("flips", C.c_int64 * 5), ("max_abs_pre", C.c_double * 5),
                ("act_abs_max", C.c_double * 5), ("act_rms", C.c_double * 5)]


class _Stats(C.Structure):
    _fields_ = [(n, C.c_double) for n in
                ("policy_loss", "entropy", "value_loss", "total_loss", "grad_norm", "clip_scale")] + \
               [("nonfinite", C.c_int32)]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_param_count.restype = C.c_uint64
        _lib.oracle_act_per_sample.restype = C.c_uint64
        _lib.oracle_sample_f32.restype = C.c_int32
        _lib.oracle_clip_f64.restype = C.c_double
        _lib.oracle_surrogate_loss_f64.restype = C.c_double
        _lib.oracle_threads.restype = C.c_int
        _lib.oracle_round_bf16.restype = C.c_double
        _lib.oracle_round_bf16.argtypes = [C.c_double]
    return _lib


def _net(net) -> _Net:
    n = _Net()
    n.in_c, n.in_h, n.in_w = net.in_c, net.in_h, net.in_w
    n.n_conv = len(net.conv)
    for i, (co, k, s) in enumerate(net.conv):
        n.conv_cout[i], n.conv_k[i], n.conv_stride[i] = co, k, s
    n.fc, n.n_actions = net.fc, net.n_actions
    n.bf16 = int(getattr(net, "bf16", 0))
    return n


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def round_bf16(v: float) -> float:
    return float(_load().oracle_round_bf16(float(v)))


def threads() -> int:
    return int(_load().oracle_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def param_count(net) -> int:
    return int(_load().oracle_param_count(C.byref(_net(net))))


def act_per_sample(net) -> int:
    return int(_load().oracle_act_per_sample(C.byref(_net(net))))


def forward_f64(net, params, states, want_acts=False):
    """states uint8 [N,C,H,W] -> (logits [N,A], values [N], acts [N,act_per_sample] or None)."""
    L = _load()
    params = _c(params, np.float64)
    states = _c(states, np.uint8)
    N = states.shape[0]
    logits = np.empty((N, net.n_actions), np.float64)
    values = np.empty(N, np.float64)
    acts = np.empty((N, act_per_sample(net)), np.float64) if want_acts else None
    L.oracle_forward_f64(C.byref(_net(net)), _p(params, C.c_double), _p(states, C.c_uint8), N,
                         _p(acts, C.c_double), _p(logits, C.c_double), _p(values, C.c_double))
    return logits, values, acts


def softmax_f64(z):
    L = _load()
    z = _c(z, np.float64)
    p = np.empty_like(z)
    lp = np.empty_like(z)
    L.oracle_softmax_f64(_p(z, C.c_double), z.size, _p(p, C.c_double), _p(lp, C.c_double))
    return p, lp


def sample_f32(p, u) -> int:
    L = _load()
    p = _c(p, np.float32)
    return int(L.oracle_sample_f32(_p(p, C.c_float), p.size, C.c_float(float(u))))


def returns_f64(rewards, dones, bootstrap, gamma):
    L = _load()
    rewards = _c(rewards, np.float32)
    dones = _c(dones, np.uint8)
    bootstrap = _c(bootstrap, np.float64)
    T, n_e = rewards.shape
    R = np.empty((T, n_e), np.float64)
    L.oracle_returns_f64(_p(rewards, C.c_float), _p(dones, C.c_uint8), _p(bootstrap, C.c_double),
                         C.c_double(gamma), T, n_e, _p(R, C.c_double))
    return R


def loss_f64(logits, values, R, actions, beta, cv, adv=None):
    """-> dict(policy_loss, entropy, value_loss, dz [B,A], dv [B])."""
    L = _load()
    logits = _c(logits, np.float64)
    B, A = logits.shape
    values = _c(values, np.float64).reshape(B)
    R = _c(R, np.float64).reshape(B)
    actions = _c(actions, np.int32).reshape(B)
    adv = _c(adv, np.float64).reshape(B) if adv is not None else None
    pl, ent, vl = C.c_double(), C.c_double(), C.c_double()
    dz = np.empty((B, A), np.float64)
    dv = np.empty(B, np.float64)
    L.oracle_loss_f64(_p(logits, C.c_double), _p(values, C.c_double), _p(R, C.c_double),
                      _p(adv, C.c_double), _p(actions, C.c_int32), B, A, C.c_double(beta),
                      C.c_double(cv), C.byref(pl), C.byref(ent), C.byref(vl),
                      _p(dz, C.c_double), _p(dv, C.c_double))
    return dict(policy_loss=pl.value, entropy=ent.value, value_loss=vl.value, dz=dz, dv=dv)


def surrogate_loss_f64(net, params, states, actions, adv, R, beta, cv) -> float:
    L = _load()
    params = _c(params, np.float64)
    states = _c(states, np.uint8)
    B = states.shape[0]
    return float(L.oracle_surrogate_loss_f64(
        C.byref(_net(net)), _p(params, C.c_double), _p(states, C.c_uint8),
        _p(_c(actions, np.int32), C.c_int32), _p(_c(adv, np.float64), C.c_double),
        _p(_c(R, np.float64), C.c_double), B, C.c_double(beta), C.c_double(cv)))


def surrogate_grad_f64(net, params, states, actions, adv, R, beta, cv):
    L = _load()
    params = _c(params, np.float64)
    states = _c(states, np.uint8)
    B = states.shape[0]
    g = np.empty(params.size, np.float64)
    L.oracle_surrogate_grad_f64(
        C.byref(_net(net)), _p(params, C.c_double), _p(states, C.c_uint8),
        _p(_c(actions, np.int32), C.c_int32), _p(_c(adv, np.float64), C.c_double),
        _p(_c(R, np.float64), C.c_double), B, C.c_double(beta), C.c_double(cv), _p(g, C.c_double))
    return g


def backward_f64(net, params, states, dz, dv):
    L = _load()
    params = _c(params, np.float64)
    states = _c(states, np.uint8)
    B = states.shape[0]
    g = np.empty(params.size, np.float64)
    L.oracle_backward_f64(C.byref(_net(net)), _p(params, C.c_double), _p(states, C.c_uint8), B,
                          _p(_c(dz, np.float64), C.c_double), _p(_c(dv, np.float64), C.c_double),
                          _p(g, C.c_double))
    return g


def clip_f64(g, c):
    """-> (clipped g, scale, norm)."""
    L = _load()
    g = np.array(g, dtype=np.float64, copy=True)
    n = C.c_double()
    s = L.oracle_clip_f64(_p(g, C.c_double), C.c_uint64(g.size), C.c_double(c), C.byref(n))
    return g, float(s), n.value


def rmsprop_f64(theta, g2, g, lr, alpha, eps):
    L = _load()
    theta = np.array(theta, dtype=np.float64, copy=True)
    g2 = np.array(g2, dtype=np.float64, copy=True)
    g = _c(g, np.float64)
    L.oracle_rmsprop_f64(_p(theta, C.c_double), _p(g2, C.c_double), _p(g, C.c_double),
                         C.c_uint64(theta.size), C.c_double(lr), C.c_double(alpha), C.c_double(eps))
    return theta, g2


def select_actions(net, params, states, uniforms, want_logits=False):
    """states uint8 [n_e,C,H,W], uniforms f32 [n_e] -> dict(actions, values, probs[, logits])."""
    L = _load()
    params = _c(params, np.float32)
    states = _c(states, np.uint8)
    uniforms = _c(uniforms, np.float32)
    n_e = states.shape[0]
    actions = np.empty(n_e, np.int32)
    values = np.empty(n_e, np.float32)
    probs = np.empty((n_e, net.n_actions), np.float32)
    logits = np.empty((n_e, net.n_actions), np.float64) if want_logits else None
    L.oracle_select_actions(C.byref(_net(net)), _p(params, C.c_float), _p(states, C.c_uint8),
                            _p(uniforms, C.c_float), n_e, _p(actions, C.c_int32),
                            _p(values, C.c_float), _p(probs, C.c_float), _p(logits, C.c_double))
    out = dict(actions=actions, values=values, probs=probs)
    if want_logits:
        out["logits"] = logits
    return out


@dataclass
class TrainResult:
    params: np.ndarray      # float32 [P] after the update
    rms: np.ndarray         # float32 [P] after the update
    grads: np.ndarray       # float64 [P] gradient before clipping
    logits: np.ndarray      # float64 [(T+1) n_e, A]
    values: np.ndarray      # float64 [(T+1) n_e]
    returns: np.ndarray     # float64 [T, n_e]
    stats: dict
    flips: dict | None = None   # masked runs: per layer (conv 1.., fc) units, flips, max_abs_pre, act_abs_max, act_rms


def train_step(net, params, rms, states, actions, rewards, dones, hp, masks=None) -> TrainResult:
    """One PAAC update.  hp: object with gamma, beta, value_coef, lr, rms_alpha, rms_eps, clip_norm.
    masks (optional): uint8 [(T+1) n_e, act_per_sample] ReLU decisions taken elsewhere, used instead of
    the oracle's own sign tests (conv outputs in NCHW order, then the fc units); the result then
    carries `flips`, the comparison with the oracle's own decisions."""
    L = _load()
    params = np.array(params, dtype=np.float32, copy=True)
    rms = np.array(rms, dtype=np.float32, copy=True)
    states = _c(states, np.uint8)
    T, n_e = states.shape[0] - 1, states.shape[1]
    actions = _c(actions, np.int32)
    rewards = _c(rewards, np.float32)
    dones = _c(dones, np.uint8)
    assert actions.shape == (T, n_e) and rewards.shape == (T, n_e) and dones.shape == (T, n_e)
    h = _HP(hp.gamma, hp.beta, hp.value_coef, hp.lr, hp.rms_alpha, hp.rms_eps, hp.clip_norm)
    st = _Stats()
    P = params.size
    grads = np.empty(P, np.float64)
    logits = np.empty(((T + 1) * n_e, net.n_actions), np.float64)
    values = np.empty((T + 1) * n_e, np.float64)
    returns = np.empty((T, n_e), np.float64)
    flips = None
    if masks is None:
        L.oracle_train_step(C.byref(_net(net)), _p(params, C.c_float), _p(rms, C.c_float),
                            _p(states, C.c_uint8), _p(actions, C.c_int32), _p(rewards, C.c_float),
                            _p(dones, C.c_uint8), C.byref(h), T, n_e, C.byref(st),
                            _p(grads, C.c_double), _p(logits, C.c_double), _p(values, C.c_double),
                            _p(returns, C.c_double))
    else:
        masks = _c(masks, np.uint8)
        assert masks.shape == ((T + 1) * n_e, act_per_sample(net)), masks.shape
        fr = _Flips()
        L.oracle_train_step_masked(C.byref(_net(net)), _p(params, C.c_float), _p(rms, C.c_float),
                                   _p(states, C.c_uint8), _p(actions, C.c_int32), _p(rewards, C.c_float),
                                   _p(dones, C.c_uint8), C.byref(h), T, n_e, _p(masks, C.c_uint8), C.byref(st),
                                   _p(grads, C.c_double), _p(logits, C.c_double), _p(values, C.c_double),
                                   _p(returns, C.c_double), C.byref(fr))
        nl = len(net.conv) + 1
        flips = {k: np.array(list(getattr(fr, k))[:nl]) for k, _ in _Flips._fields_}
    stats = {n: getattr(st, n) for n, _ in _Stats._fields_}
    return TrainResult(params, rms, grads, logits, values, returns, stats, flips)


def philox4x32_10(ctr, key):
    L = _load()
    c = (C.c_uint32 * 4)(*[int(x) for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) for x in key])
    o = (C.c_uint32 * 4)()
    L.oracle_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def fill_uniforms(seed: int, offset: int, n: int) -> np.ndarray:
    L = _load()
    out = np.empty(n, np.float32)
    L.oracle_fill_uniforms(C.c_uint64(seed), C.c_uint64(offset), _p(out, C.c_float), C.c_uint64(n))
    return out


def init_params(net, seed: int) -> np.ndarray:
    L = _load()
    out = np.empty(param_count(net), np.float32)
    L.oracle_init_params(C.byref(_net(net)), C.c_uint64(seed), _p(out, C.c_float))
    return out


# ---- value-based variant (Section 2.2) ----
def q_pick_f32(q, u, epsilon) -> int:
    L = _load()
    q = _c(q, np.float64)
    L.oracle_q_pick_f32.restype = C.c_int32
    return int(L.oracle_q_pick_f32(_p(q, C.c_double), q.size, C.c_float(float(u)), C.c_float(float(epsilon))))


def q_loss_f64(Q, R, actions, cq):
    """-> (mean squared TD error, dL/dQ [B,A]) for L = cq * mean((R - Q[a])^2)."""
    L = _load()
    Q = _c(Q, np.float64)
    B, A = Q.shape
    msq = C.c_double()
    dq = np.empty((B, A), np.float64)
    L.oracle_q_loss_f64(_p(Q, C.c_double), _p(_c(R, np.float64).reshape(B), C.c_double),
                        _p(_c(actions, np.int32).reshape(B), C.c_int32), B, A, C.c_double(cq),
                        C.byref(msq), _p(dq, C.c_double))
    return msq.value, dq


def q_surrogate_loss_f64(net, params, states, actions, R, cq) -> float:
    L = _load()
    L.oracle_q_surrogate_loss_f64.restype = C.c_double
    params = _c(params, np.float64)
    states = _c(states, np.uint8)
    return float(L.oracle_q_surrogate_loss_f64(
        C.byref(_net(net)), _p(params, C.c_double), _p(states, C.c_uint8),
        _p(_c(actions, np.int32), C.c_int32), _p(_c(R, np.float64), C.c_double), states.shape[0],
        C.c_double(cq)))


def q_surrogate_grad_f64(net, params, states, actions, R, cq):
    L = _load()
    params = _c(params, np.float64)
    states = _c(states, np.uint8)
    g = np.empty(params.size, np.float64)
    L.oracle_q_surrogate_grad_f64(
        C.byref(_net(net)), _p(params, C.c_double), _p(states, C.c_uint8),
        _p(_c(actions, np.int32), C.c_int32), _p(_c(R, np.float64), C.c_double), states.shape[0],
        C.c_double(cq), _p(g, C.c_double))
    return g


def q_select_actions(net, params, states, uniforms, epsilon):
    """-> dict(actions int32 [n_e], q float64 [n_e,A])."""
    L = _load()
    params = _c(params, np.float32)
    states = _c(states, np.uint8)
    uniforms = _c(uniforms, np.float32)
    n_e = states.shape[0]
    actions = np.empty(n_e, np.int32)
    q = np.empty((n_e, net.n_actions), np.float64)
    L.oracle_q_select_actions(C.byref(_net(net)), _p(params, C.c_float), _p(states, C.c_uint8),
                              _p(uniforms, C.c_float), n_e, C.c_float(float(epsilon)),
                              _p(actions, C.c_int32), _p(q, C.c_double))
    return dict(actions=actions, q=q)


def q_train_step(net, params, rms, states, actions, rewards, dones, hp, masks=None) -> TrainResult:
    """One update of the value-based variant; TrainResult.logits holds Q, .values is empty.
    masks: supplied ReLU decisions, as in train_step."""
    L = _load()
    params = np.array(params, dtype=np.float32, copy=True)
    rms = np.array(rms, dtype=np.float32, copy=True)
    states = _c(states, np.uint8)
    T, n_e = states.shape[0] - 1, states.shape[1]
    actions = _c(actions, np.int32)
    rewards = _c(rewards, np.float32)
    dones = _c(dones, np.uint8)
    assert actions.shape == (T, n_e) and rewards.shape == (T, n_e) and dones.shape == (T, n_e)
    h = _HP(hp.gamma, hp.beta, hp.value_coef, hp.lr, hp.rms_alpha, hp.rms_eps, hp.clip_norm)
    st = _Stats()
    grads = np.empty(params.size, np.float64)
    q = np.empty(((T + 1) * n_e, net.n_actions), np.float64)
    returns = np.empty((T, n_e), np.float64)
    flips = None
    fr = _Flips()
    if masks is not None:
        masks = _c(masks, np.uint8)
        assert masks.shape == ((T + 1) * n_e, act_per_sample(net)), masks.shape
    L.oracle_q_train_step_masked(C.byref(_net(net)), _p(params, C.c_float), _p(rms, C.c_float),
                                 _p(states, C.c_uint8), _p(actions, C.c_int32), _p(rewards, C.c_float),
                                 _p(dones, C.c_uint8), C.byref(h), T, n_e, _p(masks, C.c_uint8), C.byref(st),
                                 _p(grads, C.c_double), _p(q, C.c_double), _p(returns, C.c_double),
                                 C.byref(fr) if masks is not None else None)
    if masks is not None:
        nl = len(net.conv) + 1
        flips = {k: np.array(list(getattr(fr, k))[:nl]) for k, _ in _Flips._fields_}
    stats = {n: getattr(st, n) for n, _ in _Stats._fields_}
    return TrainResult(params, rms, grads, q, np.empty(0), returns, stats, flips)
