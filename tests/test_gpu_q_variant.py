"""GPU parity of the value-based variant (Section 2.2 on the framework of Section 3) against the
oracle: epsilon-greedy selection and the n-step Q-learning update, through the C ABI.
Tolerances as for the actor-critic path: Q values, returns and losses within 1e-4 (relative to the
tensor's largest magnitude), gradients / parameters / RMSProp state within 1e-3 relative L2; the
bf16 path within 2e-2, its gradients compared with the ReLU decisions of the HIP path handed to the
oracle.  Actions must be equal unless the two largest Q values are closer than the forward
tolerance."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_1705_04862_amd import inputs as I
from test_gpu_parity import (TOL_BF16, TOL_L2, TOL_VAL, dev, hip_relu_masks, make_ctx, rel_l2, relmax, relmax_tensor,
                             run_select, tensor_errors)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def paac():
    from paper_1705_04862_amd import paac as P
    P.lib()
    return P


def check_q_select(oracle, net, params, states, uniforms, eps, got, tol):
    acts, _, probs = got
    want = oracle.q_select_actions(net, params, states, uniforms, eps)
    q = want["q"]
    top2 = np.sort(q, axis=1)[:, -2:]
    n_guard = 0
    for e in range(states.shape[0]):
        assert 0 <= acts[e] < net.n_actions
        if acts[e] != want["actions"][e]:
            assert uniforms[e] >= eps and top2[e, 1] - top2[e, 0] < 2 * tol * np.abs(q).max(), (e, acts[e], want["actions"][e])
            n_guard += 1
    assert n_guard <= max(1, states.shape[0] // 20)
    # the distribution the kernel reports: eps/A everywhere plus 1-eps on its greedy action
    np.testing.assert_allclose(probs.sum(1), 1.0, atol=1e-5)
    greedy = probs.argmax(1)
    np.testing.assert_allclose(probs[np.arange(len(greedy)), greedy], 1 - eps + eps / net.n_actions, atol=1e-6)
    if eps < 1.0:              # at eps = 1 the distribution is flat and names no greedy action
        assert (q[np.arange(len(greedy)), greedy] >= q.max(1) - 2 * tol * np.abs(q).max()).all()


def check_q_train(oracle, net, ctx, params, rms, ro, hp, label=""):
    ctx.set_state(params, rms)
    ctx.train_step(dev(ro.states), dev(ro.actions), dev(ro.rewards), dev(ro.dones), hp)
    torch.cuda.synchronize()
    st = ctx.read_stats()
    q, _, returns = ctx.get_train_outputs()
    p2, r2, g = ctx.get_state()
    want = oracle.q_train_step(net, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, hp)
    assert relmax(q, want.logits) < TOL_VAL, label
    assert relmax(returns, want.returns) < TOL_VAL, label
    for k in ("value_loss", "total_loss", "grad_norm", "clip_scale"):
        assert abs(st[k] - want.stats[k]) <= TOL_VAL * max(abs(want.stats[k]), 1e-3) + 1e-7, (label, k, st[k], want.stats[k])
    assert st["policy_loss"] == 0 and st["entropy"] == 0 and st["nonfinite"] == 0
    assert rel_l2(g, want.grads) < TOL_L2, label
    sl = net.param_slices()
    assert not g[sl["v.W"]].any() and not g[sl["v.b"]].any()
    np.testing.assert_array_equal(p2[sl["v.W"]], params[sl["v.W"]])
    for name, s in sl.items():
        ref = want.grads[s]
        assert np.linalg.norm(g[s].astype(np.float64) - ref) <= TOL_L2 * max(np.linalg.norm(ref), 1e-3 * np.linalg.norm(want.grads)), (label, name)
    assert rel_l2(p2, want.params.astype(np.float64)) < TOL_L2, label
    assert rel_l2(p2 - params, want.params.astype(np.float64) - params) < 5 * TOL_L2, label
    assert rel_l2(r2, want.rms.astype(np.float64)) < 2 * TOL_L2, label


@pytest.mark.parametrize("ci", [0, 1, 2])
def test_q_variant_configs(paac, oracle, ci):
    cfg = I.CONFIGS[ci]
    eps = 0.25
    ctx = make_ctx(paac, cfg.net, cfg.n_e, cfg.t_max)
    ctx.set_algorithm(paac.PAAC_ALG_NSTEP_Q, eps)
    params = I.config_params(cfg, bias_range=0.05)
    rms = I.make_rms(40 + ci, cfg.net, hi=0.01)
    ctx.set_state(params)
    ro = I.config_rollout(cfg)
    for t in range(cfg.t_max):
        got = run_select(ctx, cfg.net, ro.states[t], ro.uniforms[t])
        check_q_select(oracle, cfg.net, params, ro.states[t], ro.uniforms[t], eps, got, TOL_VAL)
    check_q_train(oracle, cfg.net, ctx, params, rms, ro, cfg.hp, cfg.name)
    # switching back gives the actor-critic path again (same context, same buffers)
    ctx.set_algorithm(paac.PAAC_ALG_ACTOR_CRITIC)
    ctx.set_state(params, rms)
    ctx.train_step(dev(ro.states), dev(ro.actions), dev(ro.rewards), dev(ro.dones), cfg.hp)
    torch.cuda.synchronize()
    st = ctx.read_stats()
    want = oracle.train_step(cfg.net, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, cfg.hp)
    assert abs(st["entropy"] - want.stats["entropy"]) < TOL_VAL * want.stats["entropy"]


@pytest.mark.parametrize("net,n_e,t_max,eps", [(I.nips_net(2), 1, 1, 0.0), (I.nature_net(32), 5, 2, 1.0), (I.nips_net(7), 67, 3, 0.1),
                                               (I.nips_net(6), 2100, 1, 0.05)],
                         ids=["nips_A2_ne1_t1_greedy", "nature_A32_ne5_random", "nips_A7_ne67", "nips_ne2100_wave_per_row_kernel"])
def test_q_variant_ragged_shapes_and_extreme_epsilon(paac, oracle, net, n_e, t_max, eps):
    ctx = make_ctx(paac, net, n_e, t_max)
    ctx.set_algorithm(paac.PAAC_ALG_NSTEP_Q, eps)
    params = I.make_params(17, net, bias_range=0.1)
    rms = I.make_rms(17, net, hi=0.01)
    ctx.set_state(params)
    ro = I.make_rollout(17, net, n_e, t_max, p_done=0.3)
    got = run_select(ctx, net, ro.states[0], ro.uniforms[0])
    check_q_select(oracle, net, params, ro.states[0], ro.uniforms[0], eps, got, TOL_VAL)
    if eps == 1.0:
        want = np.minimum((ro.uniforms[0] * np.float32(net.n_actions)).astype(np.int32), net.n_actions - 1)
        np.testing.assert_array_equal(got[0], want)
    check_q_train(oracle, net, ctx, params, rms, ro, I.HParams(), "ragged")


def test_q_variant_rejects_bad_arguments(paac):
    ctx = make_ctx(paac, I.nips_net(6), 4, 2)
    for alg, eps in [(2, 0.1), (-1, 0.1), (1, 1.5), (1, -0.1), (1, float("nan"))]:
        with pytest.raises(paac.PaacError):
            ctx.set_algorithm(alg, eps)


def test_q_variant_bf16(paac, oracle):
    net, n_e, t_max, eps = I.nature_net(18), 48, 3, 0.2
    ctx = make_ctx(paac, net, n_e, t_max, 1)
    ctx.set_algorithm(paac.PAAC_ALG_NSTEP_Q, eps)
    params = I.make_params(23, net, bias_range=0.05)
    rms = I.make_rms(23, net, hi=0.01)
    ctx.set_state(params)
    ro = I.make_rollout(23, net, n_e, t_max, p_done=0.2)
    qnet = dataclasses.replace(net, bf16=1)
    got = run_select(ctx, net, ro.states[0], ro.uniforms[0])
    check_q_select(oracle, qnet, params, ro.states[0], ro.uniforms[0], eps, got, TOL_BF16)
    hp = I.HParams()
    ctx.set_state(params, rms)
    ctx.train_step(dev(ro.states), dev(ro.actions), dev(ro.rewards), dev(ro.dones), hp)
    torch.cuda.synchronize()
    st = ctx.read_stats()
    q, _, returns = ctx.get_train_outputs()
    p2, r2, g = ctx.get_state()
    # gradients with the ReLU decisions of the HIP path shared (the decision 1[pre > 0] taken in the
    # kernel's precision on both sides), every tensor at the bf16 bar
    masks = hip_relu_masks(ctx, net)
    want = oracle.q_train_step(net, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, hp)
    wq = oracle.q_train_step(qnet, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, hp, masks=masks)
    assert relmax_tensor(q, want.logits) < TOL_BF16 and relmax_tensor(returns, want.returns) < TOL_BF16
    assert abs(st["value_loss"] - want.stats["value_loss"]) <= TOL_BF16 * max(want.stats["value_loss"], 0.05)
    assert relmax_tensor(q, wq.logits) < 2e-3
    assert rel_l2(g, wq.grads) < TOL_BF16, rel_l2(g, wq.grads)
    sl = net.param_slices()
    for name, e in tensor_errors(net, g, wq.grads).items():
        if name.startswith("v."):
            continue
        assert e < TOL_BF16, (name, e)
    assert not g[sl["v.W"]].any() and not g[sl["v.b"]].any()
    assert (wq.flips["max_abs_pre"] <= 2e-3 * wq.flips["act_abs_max"]).all(), wq.flips
    assert rel_l2(p2 - params, wq.params.astype(np.float64) - params) < TOL_BF16
