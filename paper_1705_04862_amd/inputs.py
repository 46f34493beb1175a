"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This module holds configuration tables and random-number draws only: none of the
method's arithmetic (no forward pass, no returns, no losses, no optimiser) lives
here, and it imports neither the HIP binding nor the oracle.

The tensors stand in for the paper's Atari workload (Experiments, "Experimental
setup": 84x84 single-channel frames, four stacked, 8 bit): the emulator and its ROMs
are not available, so pixels are i.i.d. uniform bytes.  Rewards, dones and
hyper-parameters follow the five measurement configurations.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np


@dataclass(frozen=True)
class Net:
    """Layer list of the shared policy/value CNN (Experiments: arch_nips / arch_nature)."""

    name: str
    arch: int                      # 0 = arch_nips, 1 = arch_nature, -1 = custom (oracle only)
    in_c: int
    in_h: int
    in_w: int
    conv: Tuple[Tuple[int, int, int], ...]   # (c_out, kernel, stride), valid padding
    fc: int
    n_actions: int
    bf16: int = 0                  # 1: conv/fc weights and conv activations are stored in bf16

    def conv_out_shapes(self) -> List[Tuple[int, int, int]]:
        c, h, w = self.in_c, self.in_h, self.in_w
        out = []
        for (co, k, s) in self.conv:
            h = (h - k) // s + 1
            w = (w - k) // s + 1
            c = co
            out.append((c, h, w))
        return out

    def flat(self) -> int:
        c, h, w = self.conv_out_shapes()[-1]
        return c * h * w

    def param_shapes(self) -> List[Tuple[str, Tuple[int, ...]]]:
        """Canonical parameter order and shapes (what get/set_state exchange)."""
        shapes = []
        cin = self.in_c
        for i, (co, k, s) in enumerate(self.conv):
            shapes.append((f"conv{i + 1}.W", (co, cin, k, k)))
            shapes.append((f"conv{i + 1}.b", (co,)))
            cin = co
        shapes.append(("fc.W", (self.fc, self.flat())))
        shapes.append(("fc.b", (self.fc,)))
        shapes.append(("pi.W", (self.n_actions, self.fc)))
        shapes.append(("pi.b", (self.n_actions,)))
        shapes.append(("v.W", (self.fc,)))
        shapes.append(("v.b", (1,)))
        return shapes

    def param_count(self) -> int:
        return int(sum(int(np.prod(s)) for _, s in self.param_shapes()))

    def param_slices(self) -> Dict[str, slice]:
        off = 0
        out = {}
        for name, shp in self.param_shapes():
            n = int(np.prod(shp))
            out[name] = slice(off, off + n)
            off += n
        return out


def nips_net(n_actions: int = 6) -> Net:
    return Net("nips", 0, 4, 84, 84, ((16, 8, 4), (32, 4, 2)), 256, n_actions)


def nature_net(n_actions: int = 18) -> Net:
    return Net("nature", 1, 4, 84, 84, ((32, 8, 4), (64, 4, 2), (64, 3, 1)), 512, n_actions)


def tiny_net(n_actions: int = 3) -> Net:
    """A net small enough for finite differences over every parameter (oracle tests only)."""
    return Net("tiny", -1, 2, 20, 20, ((2, 8, 4), (3, 3, 1)), 5, n_actions)


@dataclass(frozen=True)
class HParams:
    gamma: float = 0.99
    beta: float = 0.01
    value_coef: float = 0.5
    lr: float = 0.0224
    rms_alpha: float = 0.99
    rms_eps: float = 0.1
    clip_norm: float = 3.0


@dataclass(frozen=True)
class Config:
    index: int
    net: Net
    n_e: int
    t_max: int
    precision: int                 # 0 = fp32, 1 = bf16 MFMA operands + fp32 accumulate/master
    p_done: float = 0.01
    hp: HParams = field(default_factory=HParams)

    @property
    def name(self) -> str:
        prec = "fp32" if self.precision == 0 else "bf16"
        return (f"cfg{self.index}_{self.net.name}_ne{self.n_e}_t{self.t_max}"
                f"_A{self.net.n_actions}_{prec}")


CONFIGS: Tuple[Config, ...] = (
    Config(0, nips_net(6), 4, 5, 0),
    Config(1, nips_net(6), 32, 5, 0),
    Config(2, nature_net(18), 32, 5, 0),
    Config(3, nature_net(18), 256, 5, 1),
    Config(4, nature_net(18), 1024, 20, 1, p_done=0.02),
)


def _rng(seed: int, stream: int) -> np.random.Generator:
    # one independent stream per tensor kind so that changing one shape moves no other tensor
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), int(stream)])))


def make_states(seed: int, n_slabs: int, n_e: int, net: Net) -> np.ndarray:
    """uint8 [n_slabs, n_e, C, H, W], i.i.d. uniform 0..255."""
    g = _rng(seed, 1)
    return g.integers(0, 256, size=(n_slabs, n_e, net.in_c, net.in_h, net.in_w), dtype=np.uint8)


def make_rewards(seed: int, t_max: int, n_e: int) -> np.ndarray:
    """float32 [t_max, n_e] in {-1, 0, +1} with probabilities 0.05 / 0.9 / 0.05."""
    g = _rng(seed, 2)
    u = g.random((t_max, n_e))
    r = np.zeros((t_max, n_e), dtype=np.float32)
    r[u < 0.05] = -1.0
    r[u >= 0.95] = 1.0
    return r


def make_dones(seed: int, t_max: int, n_e: int, p_done: float) -> np.ndarray:
    """uint8 [t_max, n_e], Bernoulli(p_done)."""
    g = _rng(seed, 3)
    return (g.random((t_max, n_e)) < p_done).astype(np.uint8)


def make_actions(seed: int, t_max: int, n_e: int, n_actions: int) -> np.ndarray:
    """int32 [t_max, n_e] uniform over the action set (for train-only cases)."""
    g = _rng(seed, 4)
    return g.integers(0, n_actions, size=(t_max, n_e), dtype=np.int32)


def make_uniforms(seed: int, t_max: int, n_e: int) -> np.ndarray:
    """float32 [t_max, n_e] in [0, 1) on the 2^-24 grid (the grid a 24-bit generator yields)."""
    g = _rng(seed, 5)
    k = g.integers(0, 1 << 24, size=(t_max, n_e), dtype=np.int64)
    return (k.astype(np.float64) * 2.0 ** -24).astype(np.float32)


def make_params(seed: int, net: Net, bias_range: float = 0.0) -> np.ndarray:
    """float32 [P] in canonical order.  Weights uniform in +-sqrt(6/(fan_in+fan_out))
    (the Glorot range the configurations name), biases uniform in +-bias_range
    (0 reproduces the zero-bias initial state; tests use a non-zero range so that
    a dropped bias term cannot go unnoticed)."""
    g = _rng(seed, 6)
    out = np.empty(net.param_count(), dtype=np.float32)
    off = 0
    for name, shp in net.param_shapes():
        n = int(np.prod(shp))
        if name.endswith(".W"):
            if len(shp) == 4:
                fan_in, fan_out = shp[1] * shp[2] * shp[3], shp[0] * shp[2] * shp[3]
            elif len(shp) == 2:
                fan_in, fan_out = shp[1], shp[0]
            else:
                fan_in, fan_out = shp[0], 1
            lim = float(np.sqrt(6.0 / (fan_in + fan_out)))
            out[off:off + n] = g.uniform(-lim, lim, size=n).astype(np.float32)
        else:
            out[off:off + n] = g.uniform(-bias_range, bias_range, size=n).astype(np.float32) \
                if bias_range > 0 else 0.0
        off += n
    return out


def make_rms(seed: int, net: Net, hi: float = 0.0) -> np.ndarray:
    """float32 [P] second-moment state: zeros (fresh optimiser) or uniform in [0, hi)."""
    if hi <= 0:
        return np.zeros(net.param_count(), dtype=np.float32)
    g = _rng(seed, 7)
    return g.uniform(0.0, hi, size=net.param_count()).astype(np.float32)


@dataclass
class Rollout:
    states: np.ndarray     # uint8  [t_max+1, n_e, C, H, W]; slab t_max is s_{t_max+1}
    actions: np.ndarray    # int32  [t_max, n_e]
    rewards: np.ndarray    # float32[t_max, n_e]
    dones: np.ndarray      # uint8  [t_max, n_e]
    uniforms: np.ndarray   # float32[t_max, n_e]


def make_rollout(seed: int, net: Net, n_e: int, t_max: int, p_done: float) -> Rollout:
    return Rollout(
        states=make_states(seed, t_max + 1, n_e, net),
        actions=make_actions(seed, t_max, n_e, net.n_actions),
        rewards=make_rewards(seed, t_max, n_e),
        dones=make_dones(seed, t_max, n_e, p_done),
        uniforms=make_uniforms(seed, t_max, n_e),
    )


def config_rollout(cfg: Config, k: int = 0) -> Rollout:
    """The k-th synthetic rollout of a measurement configuration (seed 1000 + index)."""
    return make_rollout(1000 + cfg.index + 7919 * k, cfg.net, cfg.n_e, cfg.t_max, cfg.p_done)


def config_params(cfg: Config, bias_range: float = 0.0) -> np.ndarray:
    return make_params(1000 + cfg.index, cfg.net, bias_range)
