"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Tolerances (fp32 path): logits, values, probabilities, returns and losses within 1e-4 of the
oracle element by element (|got - want| <= 1e-4 max(|want|, 0.05 max|want|): relative to the
element, with an absolute floor of a twentieth of the tensor's largest magnitude); gradients,
updated parameters and RMSProp state within 1e-3 relative L2 (whole vector and every tensor).
Sampled actions must be equal unless the uniform lies within 1e-5 of a CDF boundary.  Integer/bit
work (Philox, parameter initialisation, state round trips) is compared bit for bit.
bf16 path: 2e-2 everywhere (see check_train_bf16).
"""
import os

import numpy as np
import pytest
import torch

from paper_1705_04862_amd import inputs as I

pytestmark = pytest.mark.gpu

TOL_VAL = 1e-4
TOL_L2 = 1e-3


@pytest.fixture(scope="module")
def paac():
    from paper_1705_04862_amd import paac as P
    P.lib()
    return P


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


FLOOR = 0.05       # absolute floor of the element-wise check, as a fraction of the tensor's largest magnitude


def relmax(a, b):
    """Largest element-wise error relative to max(|want|, FLOOR * max|want|)."""
    b = np.asarray(b, np.float64)
    den = np.maximum(np.abs(b), FLOOR * max(np.abs(b).max(), 1e-30))
    return float((np.abs(np.asarray(a, np.float64) - b) / den).max())


def relmax_tensor(a, b):
    """Largest error relative to the tensor's largest magnitude (used where errors are absolute in
    nature: sums of many rounded bf16 terms)."""
    return float(np.abs(np.asarray(a, np.float64) - b).max() / max(np.abs(b).max(), 1e-30))


def report(line):
    """Measured figures go to the file PAAC_PARITY_REPORT names (if set) and to stdout."""
    print(line, flush=True)
    path = os.environ.get("PAAC_PARITY_REPORT")
    if path:
        with open(path, "a") as f:
            f.write(line + "\n")


def rel_l2(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - b) / max(np.linalg.norm(b), 1e-30))


def make_ctx(P, net, n_e, t_max, precision=0):
    return P.Paac(net.arch, n_e, t_max, net.n_actions, precision)


def run_select(ctx, net, states, uniforms):
    n_e = states.shape[0]
    a = torch.empty(n_e, dtype=torch.int32, device="cuda:0")
    v = torch.empty(n_e, dtype=torch.float32, device="cuda:0")
    p = torch.empty(n_e, net.n_actions, dtype=torch.float32, device="cuda:0")
    ctx.select_actions(dev(states), dev(uniforms), a, v, p)
    torch.cuda.synchronize()
    return a.cpu().numpy(), v.cpu().numpy(), p.cpu().numpy()


def check_select(oracle, net, params, states, uniforms, got):
    acts, vals, probs = got
    want = oracle.select_actions(net, params, states, uniforms)
    assert relmax(vals, want["values"].astype(np.float64)) < TOL_VAL
    assert relmax(probs, want["probs"].astype(np.float64)) < TOL_VAL
    np.testing.assert_allclose(probs.sum(1), 1.0, atol=1e-5)
    cdf = np.cumsum(want["probs"].astype(np.float64), axis=1)
    n_guard = 0
    for e in range(states.shape[0]):
        if acts[e] != want["actions"][e]:
            assert np.abs(cdf[e] - float(uniforms[e])).min() < 1e-5, (e, acts[e], want["actions"][e])
            n_guard += 1
        assert 0 <= acts[e] < net.n_actions
    assert n_guard <= max(1, states.shape[0] // 50)


def check_train(oracle, net, ctx, params, rms, ro, hp, label=""):
    """Run one train step on both sides from the same state and compare everything."""
    ctx.set_state(params, rms)
    ctx.train_step(dev(ro.states), dev(ro.actions), dev(ro.rewards), dev(ro.dones), hp)
    torch.cuda.synchronize()
    st = ctx.read_stats()
    logits, values, returns = ctx.get_train_outputs()
    p2, r2, g = ctx.get_state()
    want = oracle.train_step(net, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, hp)
    assert relmax(logits, want.logits) < TOL_VAL, label
    assert relmax(values, want.values) < TOL_VAL, label
    assert relmax(returns, want.returns) < TOL_VAL, label
    for k in ("policy_loss", "entropy", "value_loss", "total_loss", "grad_norm", "clip_scale"):
        assert abs(st[k] - want.stats[k]) <= TOL_VAL * max(abs(want.stats[k]), 1e-3) + 1e-7, (label, k, st[k], want.stats[k])
    assert st["nonfinite"] == 0
    assert rel_l2(g, want.grads) < TOL_L2, label
    for name, sl in net.param_slices().items():
        ref = want.grads[sl]
        assert np.linalg.norm(g[sl].astype(np.float64) - ref) <= TOL_L2 * max(np.linalg.norm(ref), 1e-3 * np.linalg.norm(want.grads)), (label, name)
    assert rel_l2(p2, want.params.astype(np.float64)) < TOL_L2, label
    assert rel_l2(p2 - params, want.params.astype(np.float64) - params) < 5 * TOL_L2, label     # the update itself
    assert rel_l2(r2, want.rms.astype(np.float64)) < 2 * TOL_L2, label
    return want, (p2, r2, g)


# ------------------------------------------------------------------ bit-exact pieces
def test_fill_uniforms_bit_exact(paac, oracle):
    ctx = make_ctx(paac, I.nips_net(6), 4, 5)
    for seed, off, n in [(1234, 0, 4099), (2 ** 40 + 7, 5, 1), (99, 2 ** 33, 1000), (5, 0, 3)]:
        out = torch.empty(n, dtype=torch.float32, device="cuda:0")
        ctx.fill_uniforms(seed, off, out)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out.cpu().numpy(), oracle.fill_uniforms(seed, off, n))


@pytest.mark.parametrize("net", [I.nips_net(6), I.nature_net(18)], ids=lambda n: n.name)
def test_init_params_and_state_roundtrip(paac, oracle, net):
    ctx = make_ctx(paac, net, 4, 2)
    assert ctx.param_count() == net.param_count() == oracle.param_count(net)
    ctx.init_params(42)
    p, r, _ = ctx.get_state()
    np.testing.assert_array_equal(p, oracle.init_params(net, 42))
    assert (r == 0).all()
    params = I.make_params(3, net, bias_range=0.1)
    rms = I.make_rms(3, net, hi=0.5)
    ctx.set_state(params, rms)
    p, r, _ = ctx.get_state()
    np.testing.assert_array_equal(p, params)
    np.testing.assert_array_equal(r, rms)


# ------------------------------------------------------------------ select
@pytest.mark.parametrize("ci", [0, 1, 2])
def test_select_actions_configs(paac, oracle, ci):
    cfg = I.CONFIGS[ci]
    ctx = make_ctx(paac, cfg.net, cfg.n_e, cfg.t_max)
    params = I.config_params(cfg, bias_range=0.05)
    ctx.set_state(params)
    ro = I.config_rollout(cfg)
    for t in range(cfg.t_max):
        got = run_select(ctx, cfg.net, ro.states[t], ro.uniforms[t])
        check_select(oracle, cfg.net, params, ro.states[t], ro.uniforms[t], got)


@pytest.mark.parametrize("net,n_e", [(I.nips_net(2), 1), (I.nature_net(32), 5), (I.nips_net(7), 67), (I.nature_net(4), 33),
                                     (I.nature_net(6), 100), (I.nature_net(6), 270)],
                         ids=["nips_A2_ne1", "nature_A32_ne5", "nips_A7_ne67", "nature_A4_ne33",
                              "nature_A6_ne100_one_workgroup_per_sample", "nature_A6_ne270_per_layer_exact"])
def test_select_ragged_shapes(paac, oracle, net, n_e):
    ctx = make_ctx(paac, net, n_e, 1)
    params = I.make_params(8, net, bias_range=0.1)
    ctx.set_state(params)
    st = I.make_states(8, 1, n_e, net)[0]
    u = I.make_uniforms(8, 1, n_e)[0]
    u[0] = 0.0
    u[-1] = np.float32(1.0) - np.float32(2.0 ** -24)
    check_select(oracle, net, params, st, u, run_select(ctx, net, st, u))


def test_select_extreme_pixels(paac, oracle):
    net = I.nips_net(6)
    ctx = make_ctx(paac, net, 3, 1)
    params = I.make_params(9, net, bias_range=0.1)
    ctx.set_state(params)
    st = I.make_states(9, 1, 3, net)[0]
    st[0] = 255
    st[1] = 0
    u = np.array([0.3, 0.6, 0.9], np.float32)
    check_select(oracle, net, params, st, u, run_select(ctx, net, st, u))


# ------------------------------------------------------------------ train
@pytest.mark.parametrize("ci", [0, 1, 2])
def test_train_step_configs(paac, oracle, ci):
    cfg = I.CONFIGS[ci]
    ctx = make_ctx(paac, cfg.net, cfg.n_e, cfg.t_max)
    params = I.config_params(cfg, bias_range=0.05)
    rms = I.make_rms(1000 + ci, cfg.net, hi=0.01)
    ro = I.config_rollout(cfg)
    check_train(oracle, cfg.net, ctx, params, rms, ro, cfg.hp, cfg.name)


@pytest.mark.parametrize("net,n_e,t_max,p_done", [
    (I.nips_net(3), 1, 1, 0.0), (I.nature_net(5), 3, 2, 0.5), (I.nips_net(6), 7, 20, 0.1),
    (I.nature_net(18), 2, 3, 1.0), (I.nips_net(6), 70, 2, 0.02),
    # head backward with the returns and losses computed in the same launch: an odd number of rows, the
    # longest rollout it takes (64 steps); one step more and the loss kernel runs on its own again
    (I.nature_net(5), 3, 3, 0.3), (I.nips_net(6), 2, 64, 0.1), (I.nips_net(4), 2, 65, 0.1)],
    ids=["nips_1x1", "nature_3x2", "nips_7x20", "nature_all_done", "nips_70x2", "nature_3x3", "nips_2x64", "nips_2x65"])
def test_train_ragged_and_degenerate(paac, oracle, net, n_e, t_max, p_done):
    ctx = make_ctx(paac, net, n_e, t_max)
    params = I.make_params(17, net, bias_range=0.1)
    rms = I.make_rms(17, net, hi=0.02)
    ro = I.make_rollout(17, net, n_e, t_max, p_done)
    if p_done >= 1.0:
        assert ro.dones.all()
    # clip inactive and active
    check_train(oracle, net, ctx, params, rms, ro, I.HParams(clip_norm=1e6), "noclip")
    check_train(oracle, net, ctx, params, rms, ro, I.HParams(clip_norm=0.01, lr=0.003), "clip")


def test_train_nature_above_one_sample_per_compute_unit(paac, oracle):
    """312 forward rows: more than one sample per compute unit, so the fp32 forward pass of layers 2-3
    runs in the per-layer kernels on exact bf16 parts (a workgroup walks over several samples)."""
    net = I.nature_net(6)
    ctx = make_ctx(paac, net, 52, 5)
    params = I.make_params(29, net, bias_range=0.05)
    rms = I.make_rms(29, net, hi=0.01)
    ro = I.make_rollout(29, net, 52, 5, 0.05)
    check_train(oracle, net, ctx, params, rms, ro, I.HParams(lr=0.002), "nature_52x5")


def test_train_first_step_from_zero_state_and_paper_hparams(paac, oracle):
    """Fresh optimiser state, zero biases, the paper's clipping threshold of 40."""
    cfg = I.CONFIGS[0]
    ctx = make_ctx(paac, cfg.net, cfg.n_e, cfg.t_max)
    params = I.config_params(cfg)
    ro = I.config_rollout(cfg, 1)
    check_train(oracle, cfg.net, ctx, params, I.make_rms(0, cfg.net), ro, I.HParams(clip_norm=40.0), "paper")


def test_actions_out_of_range_are_clamped(paac, oracle):
    net = I.nips_net(6)
    ctx = make_ctx(paac, net, 4, 2)
    params = I.make_params(23, net, bias_range=0.1)
    ro = I.make_rollout(23, net, 4, 2, 0.0)
    bad = ro.actions.copy()
    bad[0, 0], bad[1, 3] = -5, 99
    ro_bad = I.Rollout(ro.states, bad, ro.rewards, ro.dones, ro.uniforms)
    ctx.set_state(params)
    ctx.train_step(dev(ro_bad.states), dev(ro_bad.actions), dev(ro_bad.rewards), dev(ro_bad.dones), I.HParams())
    _, _, g = ctx.get_state()
    clamped = np.clip(bad, 0, 5)
    want = oracle.train_step(net, params, I.make_rms(0, net), ro.states, clamped, ro.rewards, ro.dones, I.HParams())
    assert rel_l2(g, want.grads) < TOL_L2


def test_multi_step_drift(paac, oracle):
    """Ten consecutive updates from the same start: optimiser state carried on both sides."""
    cfg = I.CONFIGS[0]
    net = cfg.net
    ctx = make_ctx(paac, net, cfg.n_e, cfg.t_max)
    params = I.config_params(cfg, bias_range=0.05)
    rms = I.make_rms(0, net)
    ctx.set_state(params, rms)
    op, orms = params.copy(), rms.copy()
    hp = I.HParams(lr=0.002)
    for k in range(10):
        ro = I.config_rollout(cfg, k)
        ctx.train_step(dev(ro.states), dev(ro.actions), dev(ro.rewards), dev(ro.dones), hp)
        res = oracle.train_step(net, op, orms, ro.states, ro.actions, ro.rewards, ro.dones, hp)
        op, orms = res.params, res.rms
    p, r, _ = ctx.get_state()
    assert rel_l2(p, op.astype(np.float64)) < TOL_L2
    assert rel_l2(p - params, op.astype(np.float64) - params) < 2e-2      # accumulated update
    assert rel_l2(r, orms.astype(np.float64)) < 1e-2


# ------------------------------------------------------------------ graphs, determinism, hyper-parameters
def test_graph_replay_equals_direct_launch_and_is_deterministic(paac):
    cfg = I.CONFIGS[2]
    net = cfg.net
    params = I.config_params(cfg, bias_range=0.05)
    ro = I.config_rollout(cfg)
    d = [dev(x) for x in (ro.states, ro.actions, ro.rewards, ro.dones)]
    results = []
    for graphs in (False, True, True):
        ctx = make_ctx(paac, net, cfg.n_e, cfg.t_max)
        ctx.set_graphs(graphs)
        ctx.set_state(params)
        for _ in range(3):        # with graphs on: one capture + two replays, eager work between them
            ctx.train_step(*d, cfg.hp)
            torch.cuda.synchronize()
        a = torch.empty(cfg.n_e, dtype=torch.int32, device="cuda:0")
        v = torch.empty(cfg.n_e, dtype=torch.float32, device="cuda:0")
        for _ in range(2):
            ctx.select_actions(d[0][0], dev(ro.uniforms[0]), a, v)
        torch.cuda.synchronize()
        p, r, g = ctx.get_state()
        results.append((p, r, g, a.cpu().numpy(), v.cpu().numpy(), ctx.read_stats()))
    for other in results[1:]:
        for x, y in zip(results[0][:5], other[:5]):
            np.testing.assert_array_equal(x, y)
        assert results[0][5] == other[5]


def test_hyperparameter_change_without_recapture(paac, oracle):
    cfg = I.CONFIGS[0]
    net = cfg.net
    ctx = make_ctx(paac, net, cfg.n_e, cfg.t_max)
    params = I.config_params(cfg, bias_range=0.05)
    ro = I.config_rollout(cfg)
    d = [dev(x) for x in (ro.states, ro.actions, ro.rewards, ro.dones)]
    ctx.set_state(params)
    ctx.train_step(*d, I.HParams(lr=0.01))                 # captures the graph
    ctx.set_state(params)
    hp2 = I.HParams(lr=0.0005, gamma=0.9, beta=0.1, clip_norm=0.5)
    ctx.train_step(*d, hp2)                                # replay with new hyper-parameters
    p, r, g = ctx.get_state()
    want = oracle.train_step(net, params, I.make_rms(0, net), ro.states, ro.actions, ro.rewards, ro.dones, hp2)
    assert rel_l2(g, want.grads) < TOL_L2
    assert rel_l2(p - params, want.params.astype(np.float64) - params) < 5 * TOL_L2


# ------------------------------------------------------------------ ABI robustness on the GPU
def test_error_codes(paac):
    import ctypes as C
    L = paac.lib()
    ctx = make_ctx(paac, I.nips_net(6), 4, 5)
    st = torch.zeros(4 * 28224, dtype=torch.uint8, device="cuda:0")
    u = torch.zeros(4, dtype=torch.float32, device="cuda:0")
    a = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    assert L.paac_select_actions(ctx.ctx, st.data_ptr(), u.data_ptr(), a.data_ptr(), None, None) == -5   # no params yet
    ctx.init_params(1)
    one = np.empty(16 * 400, np.float32)
    assert L.paac_get_train_activations(ctx.ctx, 0, 0, 1, one.ctypes.data_as(C.c_void_p)) == -5   # no train step yet
    assert L.paac_get_train_outputs(ctx.ctx, None, None, None) == -5
    assert L.paac_select_actions(ctx.ctx, None, u.data_ptr(), a.data_ptr(), None, None) == -1
    assert L.paac_select_actions(None, st.data_ptr(), u.data_ptr(), a.data_ptr(), None, None) == -1
    assert b"required" in L.paac_last_error(ctx.ctx)
    hp = paac.paac_hparams(0.99, 0.01, 0.5, 0.0224, 0.99, 0.1, 3.0)
    assert L.paac_train_step(ctx.ctx, None, None, None, None, C.byref(hp), None) == -1
    bad = paac.paac_hparams(1.5, 0.01, 0.5, 0.0224, 0.99, 0.1, 3.0)
    big = torch.zeros(6 * 4 * 28224, dtype=torch.uint8, device="cuda:0")
    acts = torch.zeros(20, dtype=torch.int32, device="cuda:0")
    rew = torch.zeros(20, dtype=torch.float32, device="cuda:0")
    dn = torch.zeros(20, dtype=torch.uint8, device="cuda:0")
    assert L.paac_train_step(ctx.ctx, big.data_ptr(), acts.data_ptr(), rew.data_ptr(), dn.data_ptr(), C.byref(bad), None) == -2
    # workspace too small / misaligned
    cfg = paac.paac_config(0, 4, 5, 6, 4, 84, 84, 0)
    h = C.c_void_p()
    ws = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
    assert L.paac_create(C.byref(cfg), ws.data_ptr(), 4096, None, C.byref(h)) == -3
    assert L.paac_create(C.byref(cfg), ws.data_ptr() + 4, 1 << 40, None, C.byref(h)) == -3
    assert L.paac_create(C.byref(cfg), None, 0, None, C.byref(h)) == -3
    torch.cuda.synchronize()


def test_nonfinite_flag(paac):
    cfg = I.CONFIGS[0]
    ctx = make_ctx(paac, cfg.net, cfg.n_e, cfg.t_max)
    ctx.set_state(I.config_params(cfg))
    ro = I.config_rollout(cfg)
    rew = ro.rewards.copy()
    rew[0, 0] = np.nan
    ctx.train_step(dev(ro.states), dev(ro.actions), dev(rew), dev(ro.dones), cfg.hp)
    assert ctx.read_stats()["nonfinite"] == 1


def test_profiling_mode_matches_and_reports(paac):
    cfg = I.CONFIGS[0]
    ctx = make_ctx(paac, cfg.net, cfg.n_e, cfg.t_max)
    params = I.config_params(cfg)
    ro = I.config_rollout(cfg)
    d = [dev(x) for x in (ro.states, ro.actions, ro.rewards, ro.dones)]
    ctx.set_state(params)
    ctx.train_step(*d, cfg.hp)
    ref = ctx.get_state()
    ctx.set_state(params)
    ctx.set_profiling(True)
    ctx.train_step(*d, cfg.hp)
    times = ctx.kernel_times()
    ctx.set_profiling(False)
    got = ctx.get_state()
    for x, y in zip(ref, got):
        np.testing.assert_array_equal(x, y)
    assert "train.clip_rmsprop" in times and times["train.conv1_wgrad"]["calls"] == 1
    assert all(v["ms"] > 0 for v in times.values())


# ------------------------------------------------------------------ bf16 MFMA path (precision = 1)
# bf16 operands (8 significand bits) with fp32 accumulation: everything within 2e-2 of the oracle.
TOL_BF16 = 2e-2
TOL_BF16_SAME_STORAGE = 2e-3     # forward against the oracle mode that rounds the same tensors to bf16
TOL_BF16_SAME_STORAGE_GRAD = 5e-3   # gradients against that mode with shared ReLU decisions (measured: <= 2.8e-3 at 6 samples, 1e-4..1e-3 from 100 samples on)


def hip_relu_masks(ctx, net, chunk=2048):
    """The ReLU decisions the HIP path took in its last train step: stored activation > 0, as uint8
    [(t_max+1) n_e, act_per_sample] in the oracle's order (conv outputs NCHW, then the fc units)."""
    Bp = ctx.n_e * (ctx.t_max + 1)
    per = [c * h * w for c, h, w in net.conv_out_shapes()] + [net.fc]
    masks = np.empty((Bp, sum(per)), np.uint8)
    off = 0
    for layer, n in enumerate(per):
        for r in range(0, Bp, chunk):
            rows = min(chunk, Bp - r)
            masks[r:r + rows, off:off + n] = ctx.get_train_activations(layer, n, r, rows) > 0
        off += n
    return masks


TENSOR_FLOOR = 0.05     # a tensor's error is measured against at least this fraction of the whole gradient's norm


def tensor_errors(net, g, ref, floor=TENSOR_FLOOR):
    """Per tensor: L2 error of g against ref relative to max(norm of the tensor, floor * norm of the
    whole gradient).  The floor matters for tensors that are sums with cancellation (the value head's
    bias gradient is sum_i (V_i - R_i) / B: forward errors inside the 2e-2 bar on V add up in it while
    the sum itself can be small)."""
    out = {}
    whole = np.linalg.norm(ref)
    for name, sl in net.param_slices().items():
        out[name] = float(np.linalg.norm(g[sl].astype(np.float64) - ref[sl]) / max(np.linalg.norm(ref[sl]), floor * whole, 1e-30))
    return out


def check_train_bf16(oracle, net, ctx, params, rms, ro, hp, label="", unconditioned=True, plain_masked=True):
    """One train step of the bf16 path against the oracle, everything within 2e-2.

    ReLU'(pre) = 1[pre > 0] is a binary decision taken in floating point: a unit whose pre-activation
    lies within rounding of zero can fall on either side, and one such flip moves a whole per-sample
    term of the gradient (not a rounding-sized change).  Both sides therefore take that decision in
    the same precision, the kernel's: the oracle is given the decisions the HIP path took (its stored
    activations > 0) and everything else stays the oracle's own arithmetic.  Held to 2e-2, per tensor:
      (a) forward outputs, returns and losses against the plain fp64 oracle (no masks involved);
      (b) gradients, update and RMSProp state against the fp64 oracle with the shared decisions
          (plain mode, and the mode that rounds the same tensors to bf16 as the kernels do);
      (c) every decision that differs from the oracle's own belongs to a unit whose oracle
          pre-activation is within the forward tolerance of zero (so it is a rounding flip, not an error).
    The comparison without shared decisions is reported, and bounded by what the flips themselves are
    worth in the oracle (own decisions vs supplied decisions, both computed on the CPU) plus 2e-2."""
    import dataclasses
    ctx.set_state(params, rms)
    ctx.train_step(dev(ro.states), dev(ro.actions), dev(ro.rewards), dev(ro.dones), hp)
    torch.cuda.synchronize()
    st = ctx.read_stats()
    logits, values, returns = ctx.get_train_outputs()
    p2, r2, g = ctx.get_state()
    masks = hip_relu_masks(ctx, net)
    B = ro.actions.size
    args = (ro.states, ro.actions, ro.rewards, ro.dones, hp)
    qnet = dataclasses.replace(net, bf16=1)

    # (a) forward and losses against the plain oracle
    want = oracle.train_step(net, params, rms, *args)
    assert relmax_tensor(logits, want.logits) < TOL_BF16, label
    assert relmax_tensor(values, want.values) < TOL_BF16, label
    assert relmax_tensor(returns, want.returns) < TOL_BF16, label
    scale = abs(want.stats["policy_loss"]) + hp.beta * abs(want.stats["entropy"]) + hp.value_coef * want.stats["value_loss"]
    for k in ("policy_loss", "entropy", "value_loss"):
        assert abs(st[k] - want.stats[k]) <= TOL_BF16 * max(abs(want.stats[k]), 0.05), (label, k, st[k], want.stats[k])
    assert abs(st["total_loss"] - want.stats["total_loss"]) <= TOL_BF16 * max(scale, 0.05), label
    assert st["nonfinite"] == 0

    # (b) shared ReLU decisions
    refs = [("bf16-storage oracle", oracle.train_step(qnet, params, rms, *args, masks=masks), TOL_BF16_SAME_STORAGE, TOL_BF16_SAME_STORAGE_GRAD)]
    if plain_masked:
        refs.append(("plain oracle", oracle.train_step(net, params, rms, *args, masks=masks), TOL_BF16, TOL_BF16))
    for mode, wm, tol_fwd, tol_g in refs:
        assert relmax_tensor(logits, wm.logits) < tol_fwd, (label, mode)
        assert relmax_tensor(values, wm.values) < tol_fwd, (label, mode)
        errs = tensor_errors(net, g, wm.grads)
        whole = rel_l2(g, wm.grads)
        report(f"[bf16 {label}] B={B} vs {mode}, shared ReLU decisions: whole {whole:.2e}; " +
               ", ".join(f"{k} {v:.2e}" for k, v in tensor_errors(net, g, wm.grads, 0.0).items()) + " (no floor)")
        assert whole < tol_g, (label, mode, whole)
        for name, e in errs.items():
            assert e < tol_g, (label, mode, name, e)
        assert abs(st["grad_norm"] - wm.stats["grad_norm"]) <= TOL_BF16 * wm.stats["grad_norm"], (label, mode)
        assert rel_l2(p2 - params, wm.params.astype(np.float64) - params) < TOL_BF16, (label, mode)
        assert rel_l2(r2, wm.rms.astype(np.float64)) < TOL_BF16, (label, mode)
        # (c) flips are rounding flips
        f = wm.flips
        report(f"[bf16 {label}] vs {mode}: flipped units per layer {[int(x) for x in f['flips']]} of {[int(x) for x in f['units']]}; "
               f"largest |pre| among them / largest |pre| of the layer "
               f"{[float('%.2e' % (m / a)) for m, a in zip(f['max_abs_pre'], f['act_abs_max'])]}")
        assert (f["max_abs_pre"] <= tol_fwd * f["act_abs_max"]).all(), (label, mode, f)
        assert (f["flips"] <= 0.01 * f["units"]).all(), (label, mode, f)
    # master weights stay fp32: the update is not rounded to bf16
    assert np.abs(p2 - params).max() > 0 and rel_l2(p2, refs[0][1].params.astype(np.float64)) < 1e-3

    # the comparison without shared decisions: what the flips are worth, measured in the oracle itself
    if unconditioned:
        for (mode, wm, _, _), own in zip(refs, (oracle.train_step(qnet, params, rms, *args), want)):
            budget = rel_l2(wm.grads, own.grads)
            got = rel_l2(g, own.grads)
            report(f"[bf16 {label}] vs {mode}, own decisions: {got:.2e} (the flips alone are worth {budget:.2e} in the oracle)")
            assert got <= budget + TOL_BF16, (label, mode, got, budget)
    return refs[0][1]


def check_select_bf16(oracle, net, params, states, uniforms, got):
    acts, vals, probs = got
    want = oracle.select_actions(net, params, states, uniforms)
    assert relmax_tensor(vals, want["values"].astype(np.float64)) < TOL_BF16
    assert relmax_tensor(probs, want["probs"].astype(np.float64)) < TOL_BF16
    np.testing.assert_allclose(probs.sum(1), 1.0, atol=1e-5)
    # the draw itself is exact given the kernel's own probabilities (same fp32 CDF rule)
    for e in range(states.shape[0]):
        cdf = np.cumsum(probs[e].astype(np.float32), dtype=np.float32)
        k = int(np.searchsorted(cdf, uniforms[e], side="right"))
        k = min(k, net.n_actions - 1)
        if np.abs(cdf.astype(np.float64) - float(uniforms[e])).min() > 1e-5:
            assert acts[e] == k
        # and it agrees with the oracle's draw unless bf16 error can move u across a boundary
        if acts[e] != want["actions"][e]:
            ocdf = np.cumsum(want["probs"][e].astype(np.float64))
            assert np.abs(ocdf - float(uniforms[e])).min() < TOL_BF16


@pytest.mark.parametrize("net,n_e,t_max", [(I.nips_net(6), 4, 5), (I.nature_net(18), 3, 2), (I.nature_net(18), 37, 3)],
                         ids=["nips_4x5", "nature_3x2", "nature_37x3"])
def test_bf16_small_shapes(paac, oracle, net, n_e, t_max):
    ctx = make_ctx(paac, net, n_e, t_max, precision=1)
    params = I.make_params(41, net, bias_range=0.05)
    rms = I.make_rms(41, net, hi=0.01)
    ro = I.make_rollout(41, net, n_e, t_max, 0.1)
    ctx.set_state(params, rms)
    for t in range(t_max):
        check_select_bf16(oracle, net, params, ro.states[t], ro.uniforms[t], run_select(ctx, net, ro.states[t], ro.uniforms[t]))
    check_train_bf16(oracle, net, ctx, params, rms, ro, I.HParams(), "bf16")


def test_bf16_config3_full_size(paac, oracle):
    """Configuration 3 (n_e=256, t_max=5, Nature net) at full size against the whole oracle step."""
    cfg = I.CONFIGS[3]
    assert cfg.precision == 1
    ctx = make_ctx(paac, cfg.net, cfg.n_e, cfg.t_max, precision=1)
    params = I.config_params(cfg, bias_range=0.05)
    rms = I.make_rms(1003, cfg.net, hi=0.01)
    ro = I.config_rollout(cfg)
    ctx.set_state(params, rms)
    check_select_bf16(oracle, cfg.net, params, ro.states[0], ro.uniforms[0],
                      run_select(ctx, cfg.net, ro.states[0], ro.uniforms[0]))
    check_train_bf16(oracle, cfg.net, ctx, params, rms, ro, cfg.hp, cfg.name)


def test_bf16_large_batch_per_sample_weight_gradients(paac, oracle):
    """2048 transitions (n_e=128, t_max=16, Nature net): from this batch on the weight gradients of
    layers 2-3 run in the per-sample kernel (operands transposed into LDS) instead of the tiled GEMM;
    the whole step against the oracle."""
    net = I.nature_net(6)
    n_e, t_max = 128, 16
    ctx = make_ctx(paac, net, n_e, t_max, precision=1)
    params = I.make_params(77, net, bias_range=0.05)
    rms = I.make_rms(77, net, hi=0.01)
    ro = I.make_rollout(77, net, n_e, t_max, 0.02)
    ctx.set_state(params, rms)
    check_train_bf16(oracle, net, ctx, params, rms, ro, I.HParams(), "bf16_128x16")


def test_bf16_backward_at_4096_transitions(paac, oracle):
    """4096 transitions (n_e=256, t_max=16, Nature net): the batch from which the fc data gradient runs
    on 128x128 tiles with a ragged last column tile (3136 columns), as in the largest configuration
    (whose own test additionally reaches grids that walk over more tiles than are resident at once).
    The whole step, every tensor, against the oracle."""
    net = I.nature_net(6)
    n_e, t_max = 256, 16
    ctx = make_ctx(paac, net, n_e, t_max, precision=1)
    params = I.make_params(83, net, bias_range=0.05)
    rms = I.make_rms(83, net, hi=0.01)
    ro = I.make_rollout(83, net, n_e, t_max, 0.02)
    check_train_bf16(oracle, net, ctx, params, rms, ro, I.HParams(), "bf16_256x16", unconditioned=False)


def test_bf16_per_sample_weight_gradient_with_uneven_shares(paac, oracle):
    """2100 transitions (n_e=700, t_max=3, Nature net): the smallest kind of batch that takes the per-sample
    weight-gradient kernels of layers 2-3 (from 2048 samples on), with a sample count that the workgroups
    do not share evenly: some walk over nine samples, the others over eight, so the ends of their
    pipelines (last transposition, last requests, last barrier) differ between workgroups."""
    net = I.nature_net(6)
    n_e, t_max = 700, 3
    ctx = make_ctx(paac, net, n_e, t_max, precision=1)
    params = I.make_params(89, net, bias_range=0.05)
    rms = I.make_rms(89, net, hi=0.01)
    ro = I.make_rollout(89, net, n_e, t_max, 0.02)
    check_train_bf16(oracle, net, ctx, params, rms, ro, I.HParams(), "bf16_700x3", unconditioned=False)


def test_bf16_graph_replay_deterministic(paac):
    cfg = I.CONFIGS[3]
    net = cfg.net
    ro = I.make_rollout(5, net, 16, 5, 0.02)
    params = I.make_params(5, net)
    d = [dev(x) for x in (ro.states, ro.actions, ro.rewards, ro.dones)]
    res = []
    for graphs in (False, True):
        ctx = make_ctx(paac, net, 16, 5, precision=1)
        ctx.set_graphs(graphs)
        ctx.set_state(params)
        for _ in range(3):
            ctx.train_step(*d, cfg.hp)
            torch.cuda.synchronize()
        res.append(ctx.get_state())
    for x, y in zip(res[0], res[1]):
        np.testing.assert_array_equal(x, y)


def test_bf16_config4_full_size(paac, oracle):
    """Configuration 4 (n_e=1024, t_max=20: 21504 forward rows, 20480 transitions) in the launch
    configuration bench.py times.  Select: sampled environments against the oracle.  Train step: the
    WHOLE oracle step once (bf16-storage mode, the ReLU decisions of the HIP path shared: about half
    a minute on the host's cores), every tensor of the gradient, the update and the RMSProp state at
    2e-2; forward outputs and returns additionally against the plain oracle on sampled rows."""
    import dataclasses
    cfg = I.CONFIGS[4]
    net, n_e, T = cfg.net, cfg.n_e, cfg.t_max
    qnet = dataclasses.replace(net, bf16=1)
    ctx = make_ctx(paac, net, n_e, T, precision=1)
    params = I.config_params(cfg, bias_range=0.05)
    rms = I.make_rms(1004, net, hi=0.01)
    ro = I.config_rollout(cfg)
    ctx.set_state(params, rms)
    g = np.random.default_rng(4)
    # select on one slab, 48 sampled environments
    acts, vals, probs = run_select(ctx, net, ro.states[3], ro.uniforms[3])
    es = np.sort(g.choice(n_e, 48, replace=False))
    wq = oracle.select_actions(qnet, params, ro.states[3][es], ro.uniforms[3][es])
    w0 = oracle.select_actions(net, params, ro.states[3][es], ro.uniforms[3][es])
    assert relmax_tensor(vals[es], wq["values"].astype(np.float64)) < 2e-3 and relmax_tensor(probs[es], wq["probs"].astype(np.float64)) < 2e-3
    assert relmax_tensor(vals[es], w0["values"].astype(np.float64)) < TOL_BF16 and relmax_tensor(probs[es], w0["probs"].astype(np.float64)) < TOL_BF16
    check_select_bf16(oracle, net, params, ro.states[3][es], ro.uniforms[3][es], (acts[es], vals[es], probs[es]))
    assert ((acts >= 0) & (acts < net.n_actions)).all()
    # train step at full size
    ctx.train_step(dev(ro.states), dev(ro.actions), dev(ro.rewards), dev(ro.dones), cfg.hp)
    torch.cuda.synchronize()
    st = ctx.read_stats()
    logits, values, returns = ctx.get_train_outputs()
    p2, r2, grads = ctx.get_state()
    masks = hip_relu_masks(ctx, net)
    report(f"[bf16 {cfg.name}] oracle step over {T * n_e} transitions on {oracle.threads()} threads ...")
    wm = oracle.train_step(qnet, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, cfg.hp, masks=masks)
    del masks
    assert relmax_tensor(logits, wm.logits) < TOL_BF16_SAME_STORAGE and relmax_tensor(values, wm.values) < TOL_BF16_SAME_STORAGE
    assert ro.dones.any() and relmax_tensor(returns, wm.returns) < TOL_BF16_SAME_STORAGE
    for k in ("policy_loss", "entropy", "value_loss"):
        assert abs(st[k] - wm.stats[k]) <= TOL_BF16_SAME_STORAGE * max(abs(wm.stats[k]), 0.05), (k, st[k], wm.stats[k])
    errs = tensor_errors(net, grads, wm.grads)
    whole = rel_l2(grads, wm.grads)
    report(f"[bf16 {cfg.name}] B={T * n_e} vs bf16-storage oracle, shared ReLU decisions: whole {whole:.2e}; " +
           ", ".join(f"{k} {v:.2e}" for k, v in tensor_errors(net, grads, wm.grads, 0.0).items()) + " (no floor)")
    f = wm.flips
    report(f"[bf16 {cfg.name}] flipped units per layer {[int(x) for x in f['flips']]} of {[int(x) for x in f['units']]}; largest |pre| among them / "
           f"largest |pre| of the layer {[float('%.2e' % (m / a)) for m, a in zip(f['max_abs_pre'], f['act_abs_max'])]}")
    assert whole < TOL_BF16_SAME_STORAGE_GRAD
    for name, e in errs.items():
        assert e < TOL_BF16_SAME_STORAGE_GRAD, (name, e)
    assert (f["max_abs_pre"] <= TOL_BF16_SAME_STORAGE * f["act_abs_max"]).all() and (f["flips"] <= 0.01 * f["units"]).all(), f
    assert abs(st["grad_norm"] - wm.stats["grad_norm"]) <= TOL_BF16 * wm.stats["grad_norm"]
    assert abs(st["clip_scale"] - wm.stats["clip_scale"]) <= TOL_BF16 * wm.stats["clip_scale"]
    assert rel_l2(p2 - params, wm.params.astype(np.float64) - params) < TOL_BF16
    assert rel_l2(r2, wm.rms.astype(np.float64)) < TOL_BF16
    assert st["nonfinite"] == 0
    # forward outputs and returns against the plain oracle, on rows it computes one by one
    flat_states = ro.states.reshape(-1, 4, 84, 84)
    rows = np.sort(g.choice((T + 1) * n_e, 64, replace=False))
    l0, v0, _ = oracle.forward_f64(net, params.astype(np.float64), flat_states[rows])
    assert relmax_tensor(logits[rows], l0) < TOL_BF16 and relmax_tensor(values[rows], v0) < TOL_BF16
    envs = np.sort(g.choice(n_e, 32, replace=False))
    _, vboot, _ = oracle.forward_f64(net, params.astype(np.float64), ro.states[T][envs])
    R = oracle.returns_f64(ro.rewards[:, envs], ro.dones[:, envs], vboot, cfg.hp.gamma)
    assert ro.dones[:, envs].any()
    assert np.abs(returns[:, envs] - R).max() < TOL_BF16 * max(np.abs(R).max(), 1.0)


@pytest.mark.parametrize("n_e", [16, 64, 128, 256])
def test_ne_sweep_sizes_with_scaled_learning_rate(paac, oracle, n_e):
    """Sizes of the paper's n_e study (Experiments, the n_e / learning-rate figure): lr = 0.0007 n_e,
    one select slab and one train step each, on the smaller network so the oracle stays quick."""
    net, t_max = I.nips_net(6), 5
    ctx = make_ctx(paac, net, n_e, t_max)
    params = I.make_params(300 + n_e, net, bias_range=0.05)
    rms = I.make_rms(300 + n_e, net, hi=0.01)
    ro = I.make_rollout(300 + n_e, net, n_e, t_max, 0.01)
    ctx.set_state(params, rms)
    check_select(oracle, net, params, ro.states[0], ro.uniforms[0], run_select(ctx, net, ro.states[0], ro.uniforms[0]))
    check_train(oracle, net, ctx, params, rms, ro, I.HParams(lr=0.0007 * n_e), f"ne{n_e}")


def test_heads_kernels_agree_across_the_batch_threshold(paac, oracle):
    """Up to 2048 rows the heads run one workgroup per row, above that one wavefront per row; both must
    give the oracle's answer, and the same bits for the same state."""
    net = I.nips_net(6)
    params = I.make_params(41, net, bias_range=0.1)
    st = I.make_states(41, 1, 2100, net)[0]
    u = I.make_uniforms(41, 1, 2100)[0]
    big = make_ctx(paac, net, 2100, 1)
    big.set_state(params)
    got_big = run_select(big, net, st, u)
    check_select(oracle, net, params, st, u, got_big)
    small = make_ctx(paac, net, 40, 1)
    small.set_state(params)
    got_small = run_select(small, net, st[:40], u[:40])
    assert np.array_equal(got_small[0], got_big[0][:40])
    # the conv/fc GEMMs pick other tiles and k-splits at the other batch size, so values agree to
    # rounding, not to the bit
    assert relmax_tensor(got_small[1], got_big[1][:40].astype(np.float64)) < 1e-5
    assert relmax_tensor(got_small[2], got_big[2][:40].astype(np.float64)) < 1e-5


@pytest.mark.parametrize("precision", [0, 1], ids=["fp32", "bf16"])
def test_rollout_activation_cache(paac, oracle, precision):
    """Opt-in mode: the train step reuses what the t_max select calls of the rollout computed (the
    parameters do not change in between, Algorithm 1) and runs the forward pass for the bootstrap
    states only.  Same answer as the oracle, and as the uncached step to rounding; a rollout with the
    wrong number of select calls, or a parameter reload, falls back to the full forward pass."""
    net, n_e, t_max = I.nature_net(18), 6, 4
    params = I.make_params(77, net, bias_range=0.05)
    rms = I.make_rms(77, net, hi=0.01)
    ro = I.make_rollout(77, net, n_e, t_max, 0.05)
    hp = I.HParams()
    st, ac, rw, dn = dev(ro.states), dev(ro.actions), dev(ro.rewards), dev(ro.dones)

    def rollout(ctx, n_select):
        for t in range(n_select):
            run_select(ctx, net, ro.states[t % t_max], ro.uniforms[t % t_max])

    def train(ctx):
        ctx.train_step(st, ac, rw, dn, hp)
        torch.cuda.synchronize()
        p2, r2, g = ctx.get_state()
        return p2, r2, g, ctx.get_train_outputs()

    ref = make_ctx(paac, net, n_e, t_max, precision=precision)
    ref.set_state(params, rms)
    p_ref, r_ref, g_ref, out_ref = train(ref)

    ctx = make_ctx(paac, net, n_e, t_max, precision=precision)
    ctx.set_activation_cache(True)
    # bf16: other tiles at the smaller batch move sums by fp32 rounding, which can move a stored bf16
    # value by one step and a ReLU decision with it: HIP against HIP is held to the bf16 bar only
    tol_g, tol_o = (1e-5, 1e-5) if precision == 0 else (TOL_BF16, 5e-3)
    for n_select in (t_max, t_max - 1, t_max + 2, t_max):      # cached, two fallbacks, cached again
        ctx.set_state(params, rms)
        rollout(ctx, n_select)
        p2, r2, g, out = train(ctx)
        assert rel_l2(g, g_ref) < tol_g, n_select
        assert rel_l2(p2 - params, p_ref - params) < max(tol_g, 1e-4), n_select
        for a, b in zip(out, out_ref):
            assert relmax_tensor(a, b.astype(np.float64)) < tol_o, n_select
        if n_select != t_max and precision == 0:
            assert np.array_equal(g, g_ref)                     # the fallback is the uncached path, bit for bit
    # against the oracle, cached
    ctx.set_state(params, rms)
    rollout(ctx, t_max)
    if precision == 0:
        ctx.train_step(st, ac, rw, dn, hp)
        torch.cuda.synchronize()
        want = oracle.train_step(net, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, hp)
        p2, r2, g = ctx.get_state()
        assert rel_l2(g, want.grads) < TOL_L2 and rel_l2(p2, want.params) < TOL_L2
        lg, vl, rt = ctx.get_train_outputs()
        assert relmax(lg, want.logits) < TOL_VAL and relmax(vl, want.values) < TOL_VAL and relmax(rt, want.returns) < TOL_VAL
    else:
        # the cached bf16 step against the oracle (train_step inside the check consumes the cache)
        class Cached:
            n_e, t_max = ctx.n_e, ctx.t_max

            def set_state(self, p, r):
                ctx.set_state(p, r)
                rollout(ctx, t_max)

            def __getattr__(self, name):
                return getattr(ctx, name)
        check_train_bf16(oracle, net, Cached(), params, rms, ro, hp, "bf16_cached_6x4")


@pytest.mark.gpu
def test_actor_loop_runs_algorithm_1_with_the_worker_pool():
    """Whole loop (worker pool -> upload -> select -> update) on the small configuration: the
    statistics are finite, and the result does not depend on the number of workers or on the
    activation cache beyond rounding."""
    from paper_1705_04862_amd import actor_loop as AL
    cfg = I.CONFIGS[0]
    rec = {}
    _, _, s1 = AL.run(cfg, 1, 6, 0, 6, 5, False, False, record=rec)
    _, _, s4 = AL.run(cfg, 4, 6, 0, 6, 5, False, True)
    _, _, sc = AL.run(cfg, 2, 6, 0, 6, 5, True, False)
    assert s1["nonfinite"] == 0 and np.isfinite(s1["total_loss"]) and s1["grad_norm"] > 0
    assert s1 == s4
    for k in ("policy_loss", "entropy", "value_loss", "grad_norm"):
        assert abs(s1[k] - sc[k]) <= 1e-4 * max(1.0, abs(s1[k])), (k, s1[k], sc[k])
    # the last iteration of the loop, replayed through the oracle: the actions the loop sampled from
    # the states the workers produced, then the update on that rollout
    from oracle import paac_oracle as O
    net = cfg.net
    assert rec["dones"].shape == (cfg.t_max, cfg.n_e) and rec["states"][1:].any()
    for t in range(cfg.t_max):
        sel = O.select_actions(net, rec["params"], rec["states"][t], rec["uniforms"][t])
        cdf = np.cumsum(sel["probs"].astype(np.float64), axis=1)
        for e in range(cfg.n_e):
            assert rec["actions"][t, e] == sel["actions"][e] or np.abs(cdf[e] - float(rec["uniforms"][t, e])).min() < 1e-5
    want = O.train_step(net, rec["params"], rec["rms"], rec["states"], rec["actions"], rec["rewards"], rec["dones"], cfg.hp)
    lg, vl, rt = rec["outputs"]
    assert relmax(lg, want.logits) < TOL_VAL and relmax(vl, want.values) < TOL_VAL and relmax(rt, want.returns) < TOL_VAL
    for k in ("policy_loss", "entropy", "value_loss", "total_loss", "grad_norm", "clip_scale"):
        assert abs(s1[k] - want.stats[k]) <= TOL_VAL * max(abs(want.stats[k]), 1e-3) + 1e-7, (k, s1[k], want.stats[k])
    assert rel_l2(rec["grads"], want.grads) < TOL_L2
    assert rel_l2(rec["params_after"], want.params.astype(np.float64)) < TOL_L2
    assert rel_l2(rec["rms_after"], want.rms.astype(np.float64)) < 2 * TOL_L2


@pytest.mark.parametrize("ci", [1, 2])
def test_fp32_forward_error_is_at_rounding_level(paac, oracle, ci):
    """The first layer of the fp32 path runs on the bf16 matrix cores with exact operands (bytes are
    exact in bf16, weights are three bf16 parts whose sum is the fp32 weight): the forward pass must
    stay at fp32 rounding level against the double-precision oracle, far inside the 1e-4 bar.
    (Gradients are not held to this: a ReLU unit whose pre-activation is within rounding of zero can
    take the other side than in double and moves a whole per-sample term.)"""
    cfg = I.CONFIGS[ci]
    ctx = make_ctx(paac, cfg.net, cfg.n_e, cfg.t_max)
    params = I.config_params(cfg, bias_range=0.05)
    rms = I.make_rms(1, cfg.net, hi=0.01)
    ro = I.config_rollout(cfg)
    ctx.set_state(params, rms)
    ctx.train_step(dev(ro.states), dev(ro.actions), dev(ro.rewards), dev(ro.dones), cfg.hp)
    torch.cuda.synchronize()
    logits, values, returns = ctx.get_train_outputs()
    want = oracle.train_step(cfg.net, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, cfg.hp)
    assert relmax_tensor(logits, want.logits) < 5e-6
    assert relmax_tensor(values, want.values) < 5e-6
    assert relmax_tensor(returns, want.returns) < 5e-6


@pytest.mark.parametrize("precision,net,n_e,t_max", [(0, I.nature_net(18), 32, 5), (0, I.nips_net(6), 7, 2), (0, I.nature_net(6), 40, 3),
                                                     (1, I.nature_net(18), 9, 2), (1, I.nature_net(6), 150, 1)],
                         ids=["fp32_config2", "fp32_nips_7x2", "fp32_nature_160_rows_one_workgroup_per_sample", "bf16_nature_9x2", "bf16_nature_300_rows"])
def test_stored_activations_layer_by_layer(paac, oracle, precision, net, n_e, t_max):
    """Every layer's stored output of the train step's forward pass (paac_get_train_activations)
    against the oracle's, element by element: fp32 at 1e-4; bf16 at 2e-2 against the plain oracle and at
    one bf16 step (2^-8 relative, with the 2e-3 floor of the forward check) against the oracle mode that
    rounds the same tensors.  Also the argument checks of the read-back call."""
    import dataclasses
    ctx = make_ctx(paac, net, n_e, t_max, precision=precision)
    params = I.make_params(211, net, bias_range=0.05)
    ro = I.make_rollout(211, net, n_e, t_max, 0.1)
    ctx.set_state(params)
    ctx.train_step(dev(ro.states), dev(ro.actions), dev(ro.rewards), dev(ro.dones), I.HParams())
    torch.cuda.synchronize()
    flat = ro.states.reshape(-1, net.in_c, net.in_h, net.in_w)
    _, _, want = oracle.forward_f64(net, params.astype(np.float64), flat, want_acts=True)
    wq = None
    if precision == 1:
        _, _, wq = oracle.forward_f64(dataclasses.replace(net, bf16=1), params.astype(np.float64), flat, want_acts=True)
    per = [c * h * w for c, h, w in net.conv_out_shapes()] + [net.fc]
    off = 0
    for layer, n in enumerate(per):
        got = ctx.get_train_activations(layer, n)
        assert got.shape == (flat.shape[0], n) and (got >= 0).all() and (got > 0).any()
        ref = want[:, off:off + n]
        if precision == 0:
            assert relmax(got, ref) < TOL_VAL, layer
        else:
            assert relmax_tensor(got, ref) < TOL_BF16, layer
            rq = wq[:, off:off + n]
            assert (np.abs(got - rq) <= 2.0 ** -7 * np.abs(rq) + TOL_BF16_SAME_STORAGE * np.abs(rq).max()).all(), layer
            if layer < len(net.conv):      # stored conv outputs are bf16 numbers
                np.testing.assert_array_equal(got, torch.tensor(got).to(torch.bfloat16).to(torch.float32).numpy())
        # a row range gives the same rows
        sub = ctx.get_train_activations(layer, n, 3, 2)
        np.testing.assert_array_equal(sub, got[3:5])
        off += n
    L = paac.lib()
    buf = np.empty(per[0], np.float32)
    bp = buf.ctypes.data_as(__import__("ctypes").c_void_p)
    assert L.paac_get_train_activations(ctx.ctx, len(per), 0, 1, bp) == -2          # layer out of range
    assert L.paac_get_train_activations(ctx.ctx, 0, flat.shape[0], 1, bp) == -2     # rows outside the forward batch
    assert L.paac_get_train_activations(ctx.ctx, 0, 0, 1, None) == -1
    assert L.paac_get_train_activations(ctx.ctx, 0, 0, 0, bp) == 0
