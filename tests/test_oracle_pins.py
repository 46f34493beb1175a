"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test names the passage of the paper it pins.  The paper prints no numerical example of
its own, so the pins are hand-worked cases (tests/golden), closed forms, invariants, brute
force on tiny inputs, finite differences, and torch's CPU float64 conv/linear/autograd as an
independent library on the special cases it covers.
"""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_1705_04862_amd import inputs as I

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- returns (Algorithm 1)
def _read_return_cases():
    cases = []
    for line in open(os.path.join(GOLD, "returns_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        g, r, d, v, R = [p.split() for p in line.split("|")]
        cases.append((float(g[0]), [float(x) for x in r], [int(x) for x in d], float(v[0]),
                      [float(x) for x in R]))
    return cases


@pytest.mark.parametrize("case", _read_return_cases())
def test_returns_hand_worked(oracle, case):
    gamma, r, d, v, expect = case
    R = oracle.returns_f64(np.array(r, np.float32)[:, None], np.array(d, np.uint8)[:, None],
                           np.array([v]), gamma)
    np.testing.assert_allclose(R[:, 0], expect, rtol=0, atol=1e-12)


def test_returns_closed_form_no_dones(oracle):
    """Section 4: Q^(n) = sum_{k<n} gamma^k r_{t+k} + gamma^n V(s_{t+n}), n = T - t + 1."""
    g = np.random.default_rng(0)
    T, n_e, gamma = 7, 5, 0.9
    r = g.normal(size=(T, n_e)).astype(np.float32)
    v = g.normal(size=n_e)
    R = oracle.returns_f64(r, np.zeros((T, n_e), np.uint8), v, gamma)
    for e in range(n_e):
        for t in range(T):
            n = T - t
            q = sum(gamma ** k * float(r[t + k, e]) for k in range(n)) + gamma ** n * v[e]
            assert abs(R[t, e] - q) < 1e-12


def test_returns_brute_force_with_dones(oracle):
    """With terminals: the sum stops after the first terminal transition and drops the bootstrap."""
    g = np.random.default_rng(1)
    T, n_e, gamma = 6, 40, 0.95
    r = g.normal(size=(T, n_e)).astype(np.float32)
    d = (g.random((T, n_e)) < 0.3).astype(np.uint8)
    v = g.normal(size=n_e)
    R = oracle.returns_f64(r, d, v, gamma)
    for e in range(n_e):
        for t in range(T):
            q, k, ended = 0.0, 0, False
            while t + k < T:
                q += gamma ** k * float(r[t + k, e])
                if d[t + k, e]:
                    ended = True
                    break
                k += 1
            if not ended:
                q += gamma ** (T - t) * v[e]
            assert abs(R[t, e] - q) < 1e-12
    # layout pin: time-major [t, e]; environments do not mix
    R1 = oracle.returns_f64(r[:, 3:4], d[:, 3:4], v[3:4], gamma)
    np.testing.assert_array_equal(R1[:, 0], R[:, 3])


# ---------------------------------------------------------------- softmax / entropy / sampling
@pytest.mark.parametrize("A", [6, 18])
def test_softmax_uniform_and_entropy(oracle, A):
    p, lp = oracle.softmax_f64(np.full(A, 0.37))
    np.testing.assert_allclose(p, 1.0 / A, atol=1e-15)
    np.testing.assert_allclose(lp, -math.log(A), atol=1e-14)
    H = -(p * lp).sum()
    assert abs(H - math.log(A)) < 1e-13
    assert abs(math.log(6) - 1.791759469228055) < 1e-15 and abs(math.log(18) - 2.8903717578961645) < 1e-15


def test_softmax_invariants(oracle):
    g = np.random.default_rng(2)
    for _ in range(20):
        z = g.normal(scale=5.0, size=9)
        p, lp = oracle.softmax_f64(z)
        assert abs(p.sum() - 1.0) < 1e-12
        p2, lp2 = oracle.softmax_f64(z + 123.456)
        np.testing.assert_allclose(p, p2, rtol=1e-12)
        np.testing.assert_allclose(np.exp(lp), p, rtol=1e-12)
        np.testing.assert_allclose(p, np.exp(z) / np.exp(z).sum(), rtol=1e-12)
    # large logits stay finite; one-hot limit has zero entropy
    p, lp = oracle.softmax_f64(np.array([1000.0, 0.0, -1000.0]))
    assert np.isfinite(lp).all() and abs(p[0] - 1.0) < 1e-15
    assert abs(-(p * np.where(p > 0, lp, 0)).sum()) < 1e-12


def test_sampling_inverse_cdf(oracle):
    p = np.array([0.0, 0.25, 0.5, 0.0, 0.25], np.float32)
    assert oracle.sample_f32(p, 0.0) == 1            # first action with p > 0
    assert oracle.sample_f32(p, 0.2499999) == 1
    assert oracle.sample_f32(p, 0.25) == 2           # u < cdf is strict
    assert oracle.sample_f32(p, 0.7499999) == 2
    assert oracle.sample_f32(p, 0.75) == 4
    assert oracle.sample_f32(p, np.float32(1.0) - np.float32(2.0 ** -24)) == 4
    assert oracle.sample_f32(np.array([0.3, 0.3, 0.3], np.float32), 0.95) == 2   # none -> A-1
    # monotone in u and frequencies match p
    g = np.random.default_rng(3)
    q = g.random(6).astype(np.float32)
    q /= q.sum()
    us = np.sort(g.random(20000).astype(np.float32))
    acts = np.array([oracle.sample_f32(q, u) for u in us])
    assert (np.diff(acts) >= 0).all()
    freq = np.bincount(acts, minlength=6) / len(us)
    sigma = np.sqrt(q * (1 - q) / len(us))
    assert (np.abs(freq - q) < 4.5 * sigma + 1e-6).all()


def test_entropy_gradient_values(oracle):
    """dH/dz_j = -p_j (log p_j + H): numbers worked from the formula for z = [.3,-1.2,2,.5],
    and checked against finite differences of H itself."""
    z = np.array([0.3, -1.2, 2.0, 0.5])
    out = oracle.loss_f64(z[None], np.zeros(1), np.zeros(1), np.array([0]), beta=1.0, cv=0.0)
    # with adv = R - V = 0 the policy term vanishes: dz = beta * p (log p + H) = -dH/dz
    np.testing.assert_allclose(-out["dz"][0], [0.146969, 0.075061, -0.370689, 0.148659], atol=2e-6)

    def H(zz):
        p, lp = oracle.softmax_f64(zz)
        return -(p * lp).sum()
    for j in range(4):
        e = np.zeros(4)
        e[j] = 1e-6
        fd = (H(z + e) - H(z - e)) / 2e-6
        assert abs(fd - (-out["dz"][0][j])) < 1e-8


def test_loss_terms_closed_form(oracle):
    """Section 4 batch gradients as one loss: check each term against numpy on random inputs."""
    g = np.random.default_rng(4)
    B, A = 12, 6
    z = g.normal(size=(B, A))
    v = g.normal(size=B)
    R = g.normal(size=B)
    a = g.integers(0, A, B)
    out = oracle.loss_f64(z, v, R, a, beta=0.01, cv=0.5)
    lp = z - np.log(np.exp(z).sum(1, keepdims=True))
    p = np.exp(lp)
    adv = R - v
    assert abs(out["policy_loss"] - (-(adv * lp[np.arange(B), a]).mean())) < 1e-12
    assert abs(out["entropy"] - (-(p * lp).sum(1).mean())) < 1e-12
    assert abs(out["value_loss"] - ((R - v) ** 2).mean()) < 1e-12
    np.testing.assert_allclose(out["dz"].sum(1), 0.0, atol=1e-15)       # rows of dlogits sum to 0
    np.testing.assert_allclose(out["dv"], 2 * 0.5 * (v - R) / B, rtol=1e-13)
    # beta = 0 and adv = 0  =>  no policy-head gradient at all
    out0 = oracle.loss_f64(z, R, R, a, beta=0.0, cv=0.5)
    assert np.abs(out0["dz"]).max() == 0.0


# ---------------------------------------------------------------- forward vs brute force / torch
def _split(net, params):
    sl = net.param_slices()
    return {name: np.asarray(params[sl[name]]).reshape(shp) for name, shp in net.param_shapes()}


def _torch_forward(net, params, states):
    """Independent float64 forward with torch CPU library ops."""
    p = {k: torch.tensor(v, dtype=torch.float64) for k, v in _split(net, params).items()} \
        if not isinstance(params, dict) else params
    x = torch.tensor(states.astype(np.float64)) / 255.0
    for i, (co, k, s) in enumerate(net.conv):
        x = F.relu(F.conv2d(x, p[f"conv{i + 1}.W"], p[f"conv{i + 1}.b"], stride=s))
    h = F.relu(F.linear(x.flatten(1), p["fc.W"], p["fc.b"]))
    logits = F.linear(h, p["pi.W"], p["pi.b"])
    v = F.linear(h, p["v.W"][None], p["v.b"])[:, 0]
    return logits, v


def test_shapes_and_param_counts(oracle):
    assert [s[1:] for s in I.nips_net().conv_out_shapes()] == [(20, 20), (9, 9)]
    assert [s[1:] for s in I.nature_net().conv_out_shapes()] == [(20, 20), (9, 9), (7, 7)]
    assert I.nips_net().flat() == 2592 and I.nature_net().flat() == 3136
    assert oracle.param_count(I.nips_net(6)) == 677943
    assert oracle.param_count(I.nature_net(18)) == 1693875
    assert oracle.act_per_sample(I.nature_net()) == 32 * 400 + 64 * 81 + 64 * 49 + 512


def test_conv_window_sum_and_normalisation(oracle):
    """All-ones conv weights, zero bias => first conv output = window sum of x/255 (brute force);
    byte 255 maps to exactly 1.0 and 0 to 0."""
    net = I.Net("one", -1, 2, 12, 12, ((1, 4, 2),), 3, 2)
    g = np.random.default_rng(5)
    st = g.integers(0, 256, (3, 2, 12, 12), dtype=np.uint8)
    st[0] = 255
    st[1] = 0
    P = net.param_count()
    params = np.zeros(P)
    sl = net.param_slices()
    params[sl["conv1.W"]] = 1.0
    _, _, acts = oracle.forward_f64(net, params, st, want_acts=True)
    out = acts[:, :25].reshape(3, 5, 5)
    assert (out[0] == 32.0).all() and (out[1] == 0.0).all()
    x = st[2].astype(np.float64) / 255.0
    for oy in range(5):
        for ox in range(5):
            assert abs(out[2, oy, ox] - x[:, oy * 2:oy * 2 + 4, ox * 2:ox * 2 + 4].sum()) < 1e-12


@pytest.mark.parametrize("net", [I.nips_net(6), I.nature_net(18), I.tiny_net(3)], ids=lambda n: n.name)
def test_forward_matches_torch_f64(oracle, net):
    params = I.make_params(11, net, bias_range=0.1).astype(np.float64)
    st = I.make_states(11, 1, 3, net)[0]
    logits, values, acts = oracle.forward_f64(net, params, st, want_acts=True)
    tl, tv = _torch_forward(net, params, st)
    np.testing.assert_allclose(logits, tl.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(values, tv.numpy(), rtol=1e-11, atol=1e-12)
    assert (acts >= 0).all() and (acts == 0).any()      # ReLU really clips something


# ---------------------------------------------------------------- gradients
def _fd_case(seed=21):
    net = I.tiny_net(3)
    g = np.random.default_rng(seed)
    B = 6
    st = g.integers(0, 256, (B, net.in_c, net.in_h, net.in_w), dtype=np.uint8)
    params = I.make_params(seed, net, bias_range=0.2).astype(np.float64)
    a = g.integers(0, 3, B).astype(np.int32)
    adv = g.normal(size=B)
    R = g.normal(size=B)
    return net, params, st, a, adv, R


def test_gradient_finite_differences(oracle):
    """Every parameter of a tiny net: analytic backward vs central differences in fp64 of the
    scalar whose gradient Section 4 / Algorithm 1 (the d-theta lines) follow."""
    net, params, st, a, adv, R = _fd_case()
    beta, cv = 0.05, 0.5
    g = oracle.surrogate_grad_f64(net, params, st, a, adv, R, beta, cv)
    fd = np.empty_like(g)
    h = 1e-6
    for i in range(params.size):
        pp = params.copy(); pp[i] += h
        pm = params.copy(); pm[i] -= h
        fd[i] = (oracle.surrogate_loss_f64(net, pp, st, a, adv, R, beta, cv) -
                 oracle.surrogate_loss_f64(net, pm, st, a, adv, R, beta, cv)) / (2 * h)
    assert np.abs(g).max() > 1e-3
    err = np.abs(g - fd) / np.maximum(1e-3 * np.abs(g).max(), np.abs(fd))
    assert err.max() < 1e-5, err.max()
    # every tensor carries signal (a dropped layer gradient would be all zeros)
    for name, s in net.param_slices().items():
        assert np.abs(g[s]).max() > 0, name


@pytest.mark.parametrize("net", [I.tiny_net(3), I.nips_net(6)], ids=lambda n: n.name)
def test_gradient_matches_torch_autograd(oracle, net):
    g = np.random.default_rng(31)
    B = 4
    st = g.integers(0, 256, (B, net.in_c, net.in_h, net.in_w), dtype=np.uint8)
    params = I.make_params(31, net, bias_range=0.1).astype(np.float64)
    a = g.integers(0, net.n_actions, B).astype(np.int32)
    adv = g.normal(size=B)
    R = g.normal(size=B)
    beta, cv = 0.01, 0.5
    got = oracle.surrogate_grad_f64(net, params, st, a, adv, R, beta, cv)
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in _split(net, params).items()}
    logits, v = _torch_forward(net, tp, st)
    lp = F.log_softmax(logits, dim=1)
    H = -(lp.exp() * lp).sum(1)
    loss = (-(torch.tensor(adv) * lp[torch.arange(B), torch.tensor(a, dtype=torch.long)]).mean()
            - beta * H.mean() + cv * ((torch.tensor(R) - v) ** 2).mean())
    loss.backward()
    want = np.concatenate([tp[name].grad.numpy().ravel() for name, _ in net.param_shapes()])
    np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-13)
    assert abs(oracle.surrogate_loss_f64(net, params, st, a, adv, R, beta, cv) - loss.item()) < 1e-12


# ---------------------------------------------------------------- clip / RMSProp
def test_clip_pins(oracle):
    g, s, n = oracle.clip_f64([60.0, 80.0], 40.0)          # ||g|| = 100 -> scale 0.4
    np.testing.assert_allclose(g, [24.0, 32.0], rtol=1e-15)
    assert abs(s - 0.4) < 1e-15 and abs(n - 100.0) < 1e-12
    x = np.random.default_rng(6).normal(size=1000)
    y, s, n = oracle.clip_f64(x, 1e3)                       # below the threshold: untouched bits
    assert s == 1.0 and (y == x).all() and abs(n - np.linalg.norm(x)) < 1e-10
    y, s, n = oracle.clip_f64(x, 3.0)
    assert abs(np.linalg.norm(y) - 3.0) < 1e-12
    y, s, n = oracle.clip_f64(np.zeros(5), 3.0)
    assert s == 1.0 and n == 0.0


def test_rmsprop_pins(oracle):
    """First step from zero state: theta' = theta - lr g / sqrt((1-a) g^2 + eps), eps inside the root
    (hyper-parameters of the Experiments section: lr .0224, decay .99, eps .1)."""
    th, g2 = oracle.rmsprop_f64([1.0], [0.0], [2.0], 0.0224, 0.99, 0.1)
    assert abs(g2[0] - 0.04) < 1e-15
    assert abs(th[0] - (1.0 - 0.0224 * 2.0 / math.sqrt(0.14))) < 1e-15
    assert abs(th[0] - 0.8802670) < 1e-6
    th, g2 = oracle.rmsprop_f64([1.0], [0.5], [0.0], 0.0224, 0.99, 0.1)   # zero gradient
    assert th[0] == 1.0 and abs(g2[0] - 0.495) < 1e-15
    th, g2 = oracle.rmsprop_f64([0.0, 0.0], [0.0, 0.0], [1e6, -1e6], 0.0224, 0.99, 0.1)
    np.testing.assert_allclose(th, [-0.224, 0.224], rtol=1e-6)             # lr / sqrt(1 - a)
    # eps outside the root would give 1 - .0224*2/(.2+.1) = .85067: make sure that is not what we do
    th, _ = oracle.rmsprop_f64([1.0], [0.0], [2.0], 0.0224, 0.99, 0.1)
    assert abs(th[0] - 0.85067) > 0.02


# ---------------------------------------------------------------- whole step, by composition
def test_train_step_composition_against_torch(oracle):
    """One full update on the tiny net: returns, advantage (no gradient through it), three losses,
    backward, clip before RMSProp -- rebuilt here with torch float64 autograd and numpy."""
    net = I.tiny_net(3)
    T, n_e = 3, 4
    ro = I.make_rollout(77, net, n_e, T, p_done=0.3)
    assert ro.dones.any()
    params = I.make_params(77, net, bias_range=0.2)
    rms = I.make_rms(77, net, hi=0.02)
    hp = I.HParams(clip_norm=0.05)
    res = oracle.train_step(net, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, hp)

    B = T * n_e
    tp = {k: torch.tensor(v.astype(np.float64), requires_grad=True) for k, v in _split(net, params).items()}
    logits, v = _torch_forward(net, tp, ro.states.reshape(-1, net.in_c, net.in_h, net.in_w))
    vd = v.detach().numpy()
    R = np.zeros((T, n_e))
    nxt = vd[B:].copy()
    for t in range(T - 1, -1, -1):
        nxt = ro.rewards[t].astype(np.float64) + hp.gamma * (1 - ro.dones[t]) * nxt
        R[t] = nxt
    np.testing.assert_allclose(res.returns, R, rtol=1e-12, atol=1e-13)
    Rt = torch.tensor(R.ravel())
    adv = Rt - v[:B].detach()
    lp = F.log_softmax(logits[:B], dim=1)
    act = torch.tensor(ro.actions.ravel(), dtype=torch.long)
    pl = -(adv * lp[torch.arange(B), act]).mean()
    ent = -(lp.exp() * lp).sum(1).mean()
    vl = ((Rt - v[:B]) ** 2).mean()
    loss = pl - hp.beta * ent + hp.value_coef * vl
    loss.backward()
    g = np.concatenate([tp[name].grad.numpy().ravel() for name, _ in net.param_shapes()])
    np.testing.assert_allclose(res.grads, g, rtol=1e-9, atol=1e-13)
    assert abs(res.stats["policy_loss"] - pl.item()) < 1e-12
    assert abs(res.stats["entropy"] - ent.item()) < 1e-12
    assert abs(res.stats["value_loss"] - vl.item()) < 1e-12
    assert abs(res.stats["total_loss"] - loss.item()) < 1e-12
    n = np.linalg.norm(g)
    assert n > hp.clip_norm                       # the clip is active in this case
    assert abs(res.stats["grad_norm"] - n) < 1e-12 and abs(res.stats["clip_scale"] - hp.clip_norm / n) < 1e-12
    gc = g * hp.clip_norm / n
    g2 = hp.rms_alpha * rms.astype(np.float64) + (1 - hp.rms_alpha) * gc * gc
    th = params.astype(np.float64) - hp.lr * gc / np.sqrt(g2 + hp.rms_eps)
    np.testing.assert_array_equal(res.rms, g2.astype(np.float32))
    np.testing.assert_array_equal(res.params, th.astype(np.float32))


def test_select_actions_composition(oracle):
    net = I.nips_net(6)
    params = I.make_params(5, net, bias_range=0.1)
    st = I.make_states(5, 1, 8, net)[0]
    u = I.make_uniforms(5, 1, 8)[0]
    out = oracle.select_actions(net, params, st, u, want_logits=True)
    logits, values, _ = oracle.forward_f64(net, params.astype(np.float64), st)
    np.testing.assert_array_equal(out["logits"], logits)
    np.testing.assert_array_equal(out["values"], values.astype(np.float32))
    for e in range(8):
        p, _ = oracle.softmax_f64(logits[e])
        np.testing.assert_array_equal(out["probs"][e], p.astype(np.float32))
        cdf = np.cumsum(p)
        a = int(np.searchsorted(cdf, u[e], side="right"))
        if np.abs(cdf - u[e]).min() > 1e-6:
            assert out["actions"][e] == min(a, 5)


# ---------------------------------------------------------------- Philox / init
def test_philox_known_answers(oracle):
    for line in open(os.path.join(GOLD, "philox_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        c, k, o = [[int(w, 16) for w in part.split()] for part in line.split("|")]
        assert oracle.philox4x32_10(c, k) == o


def test_fill_uniforms(oracle):
    u = oracle.fill_uniforms(1234, 0, 4099)
    assert u.dtype == np.float32 and (u >= 0).all() and (u < 1).all()
    assert (u * 2 ** 24 == np.round(u * 2 ** 24)).all()
    # stream position semantics: offset counts blocks of four
    np.testing.assert_array_equal(oracle.fill_uniforms(1234, 5, 40), u[20:60])
    w = oracle.philox4x32_10([7, 0, 0, 0], [1234, 0])
    np.testing.assert_array_equal(u[28:32], [np.float32((x >> 8) * 2.0 ** -24) for x in w])
    big = oracle.fill_uniforms(99, 0, 200000)
    assert abs(big.mean() - 0.5) < 4 / math.sqrt(12 * 200000) and abs(big.var() - 1 / 12) < 1e-3
    assert not np.array_equal(oracle.fill_uniforms(100, 0, 16), big[:16])


def test_init_params_glorot(oracle):
    net = I.nature_net(18)
    p = oracle.init_params(net, 42)
    np.testing.assert_array_equal(p, oracle.init_params(net, 42))
    assert not np.array_equal(p, oracle.init_params(net, 43))
    for name, shp in net.param_shapes():
        x = p[net.param_slices()[name]]
        if name.endswith(".b"):
            assert (x == 0).all()
            continue
        if len(shp) == 4:
            fi, fo = shp[1] * shp[2] * shp[3], shp[0] * shp[2] * shp[3]
        elif len(shp) == 2:
            fi, fo = shp[1], shp[0]
        else:
            fi, fo = shp[0], 1
        lim = math.sqrt(6.0 / (fi + fo))
        assert np.abs(x).max() <= lim * (1 + 1e-6)
        if x.size > 5000:
            assert np.abs(x).max() > 0.99 * lim
            assert abs(x.mean()) < 5 * lim / math.sqrt(3 * x.size)
            assert abs(x.var() - lim * lim / 3) < 0.05 * lim * lim / 3


# ---------------------------------------------------------------- bf16 storage emulation
def test_round_bf16_matches_library_and_known_values(oracle):
    """Round-to-nearest-even to 8 significand bits: hand values and torch's CPU bfloat16 cast."""
    assert oracle.round_bf16(1.0) == 1.0
    assert oracle.round_bf16(1 + 2 ** -8) == 1.0                 # tie -> even
    assert oracle.round_bf16(1 + 3 * 2 ** -8) == 1 + 2 ** -6     # tie -> even (up)
    assert oracle.round_bf16(1 + 2 ** -8 + 2 ** -20) == 1 + 2 ** -7
    assert oracle.round_bf16(-3.14159) == -3.140625
    for b in range(256):                                          # every byte value is exact in bf16
        assert oracle.round_bf16(float(b)) == float(b)
    g = np.random.default_rng(7)
    x = np.concatenate([g.normal(size=2000), g.normal(size=2000) * 1e-6, g.normal(size=2000) * 1e6]).astype(np.float32)
    want = torch.tensor(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.round_bf16(float(v)) for v in x], np.float32)
    np.testing.assert_array_equal(got, want)


def test_bf16_storage_mode_of_the_oracle(oracle):
    """The storage-emulating mode rounds exactly the documented tensors: conv activations come out
    on the bf16 grid, the fc output and the heads do not; its forward stays within bf16 error of
    the plain oracle; and it equals a torch float64 forward with the same roundings."""
    import dataclasses
    net = I.nature_net(18)
    qnet = dataclasses.replace(net, bf16=1)
    params = I.make_params(12, net, bias_range=0.05).astype(np.float64)
    st = I.make_states(12, 1, 2, net)[0]
    lq, vq, aq = oracle.forward_f64(qnet, params, st, want_acts=True)
    l0, v0, _ = oracle.forward_f64(net, params, st)
    n_conv_act = 32 * 400 + 64 * 81 + 64 * 49
    conv_acts = aq[:, :n_conv_act].astype(np.float32)
    np.testing.assert_array_equal(conv_acts, torch.tensor(conv_acts).to(torch.bfloat16).to(torch.float32).numpy())
    h = aq[:, n_conv_act:].astype(np.float32)
    assert (h != torch.tensor(h).to(torch.bfloat16).to(torch.float32).numpy()).any()
    assert 0 < np.abs(lq - l0).max() < 2e-2 * np.abs(l0).max()
    # torch float64 with the same rounding points
    q = lambda t: t.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    P = {k: torch.tensor(v) for k, v in _split(net, params).items()}
    x = torch.tensor(st.astype(np.float64)) / 255.0
    for i, (co, k, s) in enumerate(net.conv):
        x = q(F.relu(F.conv2d(x, q(P[f"conv{i + 1}.W"]), P[f"conv{i + 1}.b"], stride=s)))
    hh = F.relu(F.linear(x.flatten(1), q(P["fc.W"]), P["fc.b"]))
    lt = F.linear(hh, P["pi.W"], P["pi.b"]).numpy()
    assert np.abs(lq - lt).max() < 2e-3 * np.abs(lt).max()        # same roundings up to ties met from either side


# ---------------------------------------------------------------- bf16 storage emulation, backward
class _RoundGrad(torch.autograd.Function):
    """Identity whose incoming gradient is rounded to bf16 (a gradient stored in bf16 between layers)."""

    @staticmethod
    def forward(ctx, x):
        return x.view_as(x)

    @staticmethod
    def backward(ctx, g):
        return g.to(torch.float32).to(torch.bfloat16).to(torch.float64)


class _RoundValue(torch.autograd.Function):
    """Rounds the value to bf16 and passes the gradient through (a tensor stored in bf16; the master
    copy it was rounded from receives the gradient unchanged)."""

    @staticmethod
    def forward(ctx, x):
        return x.to(torch.float32).to(torch.bfloat16).to(torch.float64)

    @staticmethod
    def backward(ctx, g):
        return g


def _torch_bf16_storage_step(net, params, ro, hp, round_conv_grads=True, round_fc_grad=True):
    """Section 4's loss on a network with bf16 storage points, by torch float64 autograd: conv and fc
    weights as used and conv outputs rounded to bf16; the gradient entering every ReLU layer (conv
    layers and the fc layer) rounded to bf16 after the ReLU mask; everything else in double."""
    T, n_e = ro.actions.shape
    B = T * n_e
    tp = {k: torch.tensor(v.astype(np.float64), requires_grad=True) for k, v in _split(net, params).items()}
    x = torch.tensor(ro.states.reshape(-1, net.in_c, net.in_h, net.in_w).astype(np.float64)) / 255.0
    for i, (co, k, s) in enumerate(net.conv):
        pre = F.conv2d(x, _RoundValue.apply(tp[f"conv{i + 1}.W"]), tp[f"conv{i + 1}.b"], stride=s)
        if round_conv_grads:
            pre = _RoundGrad.apply(pre)
        x = _RoundValue.apply(F.relu(pre))
    pre = F.linear(x.flatten(1), _RoundValue.apply(tp["fc.W"]), tp["fc.b"])
    if round_fc_grad:
        pre = _RoundGrad.apply(pre)
    h = F.relu(pre)
    logits = F.linear(h, tp["pi.W"], tp["pi.b"])
    v = F.linear(h, tp["v.W"][None], tp["v.b"])[:, 0]
    vd = v.detach().numpy()
    R = np.zeros((T, n_e))
    nxt = vd[B:].copy()
    for t in range(T - 1, -1, -1):
        nxt = ro.rewards[t].astype(np.float64) + hp.gamma * (1 - ro.dones[t]) * nxt
        R[t] = nxt
    Rt = torch.tensor(R.ravel())
    lp = F.log_softmax(logits[:B], dim=1)
    act = torch.tensor(ro.actions.ravel(), dtype=torch.long)
    loss = (-((Rt - v[:B].detach()) * lp[torch.arange(B), act]).mean() + hp.beta * (lp.exp() * lp).sum(1).mean()
            + hp.value_coef * ((Rt - v[:B]) ** 2).mean())
    loss.backward()
    return np.concatenate([tp[name].grad.numpy().ravel() for name, _ in net.param_shapes()]), logits.detach().numpy()


@pytest.mark.parametrize("net,n_e,T", [(I.tiny_net(3), 4, 3), (I.nature_net(18), 2, 1)], ids=["tiny", "nature"])
def test_bf16_storage_backward_of_the_oracle(oracle, net, n_e, T):
    """The backward pass of the storage-emulating mode: the gradient handed from layer to layer is
    rounded to bf16 where it enters a ReLU layer (after the mask), weights as used are the rounded
    ones, their gradient goes to the master copy.  Rebuilt with torch float64 autograd and explicit
    rounding hooks; moving or dropping a rounding point is detected."""
    import dataclasses
    qnet = dataclasses.replace(net, bf16=1)
    ro = I.make_rollout(91, net, n_e, T, p_done=0.2)
    params = I.make_params(91, net, bias_range=0.1)
    hp = I.HParams(clip_norm=1e9)
    res = oracle.train_step(qnet, params, I.make_rms(0, net), ro.states, ro.actions, ro.rewards, ro.dones, hp)
    want, logits = _torch_bf16_storage_step(net, params, ro, hp)
    # forward first: only then is the backward comparison meaningful (no rounding tie met from the other side)
    np.testing.assert_allclose(res.logits, logits, rtol=1e-9, atol=1e-12)
    scale = np.abs(want).max()
    np.testing.assert_allclose(res.grads, want, rtol=1e-8, atol=1e-11 * scale)
    for name, sl in net.param_slices().items():
        assert np.abs(want[sl]).max() > 0, name
    # the rounding points matter at the 2^-9 level and the pin sees each of them
    for kw in (dict(round_conv_grads=False), dict(round_fc_grad=False)):
        other, _ = _torch_bf16_storage_step(net, params, ro, hp, **kw)
        rel = np.linalg.norm(other - res.grads) / np.linalg.norm(res.grads)
        assert 1e-5 < rel < 2e-2, (kw, rel)
    plain = oracle.train_step(net, params, I.make_rms(0, net), ro.states, ro.actions, ro.rewards, ro.dones, hp)
    assert np.linalg.norm(plain.grads - res.grads) > 1e-5 * np.linalg.norm(res.grads)


# ---------------------------------------------------------------- supplied ReLU decisions
def _own_masks(oracle, net, params, states):
    _, _, acts = oracle.forward_f64(net, params.astype(np.float64), states.reshape(-1, net.in_c, net.in_h, net.in_w),
                                    want_acts=True)
    return (acts > 0).astype(np.uint8)


def test_supplied_relu_decisions_equal_to_own_change_nothing(oracle):
    net = I.nips_net(6)
    ro = I.make_rollout(13, net, 3, 2, p_done=0.3)
    params = I.make_params(13, net, bias_range=0.1)
    rms = I.make_rms(13, net, hi=0.02)
    hp = I.HParams()
    a = oracle.train_step(net, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, hp)
    m = _own_masks(oracle, net, params, ro.states)
    b = oracle.train_step(net, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, hp, masks=m)
    for x, y in ((a.grads, b.grads), (a.logits, b.logits), (a.values, b.values), (a.returns, b.returns),
                 (a.params, b.params), (a.rms, b.rms)):
        np.testing.assert_array_equal(x, y)
    assert a.stats == b.stats
    assert (b.flips["flips"] == 0).all()
    shapes = net.conv_out_shapes()
    assert list(b.flips["units"]) == [9 * c * h * w for c, h, w in shapes] + [9 * net.fc]
    assert (b.flips["act_rms"] > 0).all() and (b.flips["act_abs_max"] >= b.flips["act_rms"]).all()


def test_supplied_relu_decisions_against_torch_autograd(oracle):
    """Arbitrary (random) decisions: the network becomes x -> m * pre per layer, whose gradient torch's
    float64 autograd gives directly; the flip report counts the units that differ from the sign test
    and the largest pre-activation among them."""
    net = I.tiny_net(3)
    T, n_e = 2, 3
    B, Bp = T * n_e, (T + 1) * n_e
    ro = I.make_rollout(55, net, n_e, T, p_done=0.2)
    params = I.make_params(55, net, bias_range=0.2)
    hp = I.HParams(clip_norm=1e9)
    g = np.random.default_rng(55)
    masks = (g.random((Bp, oracle.act_per_sample(net))) < 0.6).astype(np.uint8)
    res = oracle.train_step(net, params, I.make_rms(0, net), ro.states, ro.actions, ro.rewards, ro.dones, hp, masks=masks)

    tp = {k: torch.tensor(v.astype(np.float64), requires_grad=True) for k, v in _split(net, params).items()}
    x = torch.tensor(ro.states.reshape(-1, net.in_c, net.in_h, net.in_w).astype(np.float64)) / 255.0
    off, n_flip, max_pre = 0, [], []
    for i, (co, k, s) in enumerate(net.conv):
        pre = F.conv2d(x, tp[f"conv{i + 1}.W"], tp[f"conv{i + 1}.b"], stride=s)
        n = pre[0].numel()
        m = torch.tensor(masks[:, off:off + n].reshape(pre.shape).astype(np.float64))
        off += n
        d = (m.numpy() > 0) != (pre.detach().numpy() > 0)
        n_flip.append(int(d.sum()))
        max_pre.append(float(np.abs(pre.detach().numpy())[d].max()))
        x = m * pre
    pre = F.linear(x.flatten(1), tp["fc.W"], tp["fc.b"])
    m = torch.tensor(masks[:, off:].astype(np.float64))
    d = (m.numpy() > 0) != (pre.detach().numpy() > 0)
    n_flip.append(int(d.sum()))
    max_pre.append(float(np.abs(pre.detach().numpy())[d].max()))
    h = m * pre
    logits = F.linear(h, tp["pi.W"], tp["pi.b"])
    v = F.linear(h, tp["v.W"][None], tp["v.b"])[:, 0]
    np.testing.assert_allclose(res.logits, logits.detach().numpy(), rtol=1e-10, atol=1e-12)
    R = torch.tensor(res.returns.ravel())
    lp = F.log_softmax(logits[:B], dim=1)
    act = torch.tensor(ro.actions.ravel(), dtype=torch.long)
    loss = (-((R - v[:B].detach()) * lp[torch.arange(B), act]).mean() + hp.beta * (lp.exp() * lp).sum(1).mean()
            + hp.value_coef * ((R - v[:B]) ** 2).mean())
    loss.backward()
    want = np.concatenate([tp[name].grad.numpy().ravel() for name, _ in net.param_shapes()])
    np.testing.assert_allclose(res.grads, want, rtol=1e-9, atol=1e-13)
    assert list(res.flips["flips"]) == n_flip and min(n_flip) > 0
    np.testing.assert_allclose(res.flips["max_abs_pre"], max_pre, rtol=1e-10)
