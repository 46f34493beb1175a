"""Host worker pool + synthetic environment (paper Section 3, Algorithm 1: n_e environments stepped by
n_w workers).  CPU only: determinism across worker counts, frame stacking, episode restarts, reward
and termination statistics, argument checks."""
import ctypes as C

import numpy as np
import pytest

from paper_1705_04862_amd import actors as A

OBS = (4, 84, 84)


def rollout(n_e, n_w, steps, seed=3, p_done=0.05, sprites=6, action_seed=11):
    env = A.Actors(n_e, n_w, seed=seed, p_done=p_done, sprites=sprites)
    s = np.zeros((n_e,) + OBS, np.uint8)
    r = np.zeros(n_e, np.float32)
    d = np.zeros(n_e, np.uint8)
    env.reset(s)
    rng = np.random.default_rng(action_seed)
    out = [(s.copy(), None, None, None)]
    for _ in range(steps):
        a = rng.integers(0, 6, n_e).astype(np.int32)
        env.step(a, s, r, d)
        out.append((s.copy(), r.copy(), d.copy(), a))
    env.close()
    return out


def test_library_exports_every_declared_symbol():
    L = A.lib()
    for name in A.SYMBOLS:
        assert hasattr(L, name), name
    import re, os
    hdr = open(os.path.join(os.path.dirname(__file__), "..", "include", "paac_actors.h")).read()
    declared = set(re.findall(r"\b(paac_actors_\w+)\s*\(", hdr))
    assert declared == set(A.SYMBOLS)


@pytest.mark.parametrize("n_w", [2, 3, 8, 16])
def test_results_do_not_depend_on_the_number_of_workers(n_w):
    ref = rollout(16, 1, 40)
    got = rollout(16, n_w, 40)
    for (s0, r0, d0, _), (s1, r1, d1, _) in zip(ref, got):
        assert np.array_equal(s0, s1)
        if r0 is not None:
            assert np.array_equal(r0, r1) and np.array_equal(d0, d1)


def test_reset_gives_three_black_frames_and_one_rendered():
    s = rollout(5, 2, 0)[0][0]
    assert not s[:, :3].any()
    assert (s[:, 3] != 0).any(axis=(1, 2)).all()
    # environments differ from each other
    assert not np.array_equal(s[0, 3], s[1, 3])


def test_frames_shift_by_one_and_restart_after_done():
    tr = rollout(8, 4, 60, p_done=0.1)
    n_done = 0
    for (sp, *_), (sn, r, d, a) in zip(tr[:-1], tr[1:]):
        for e in range(8):
            if d[e]:
                n_done += 1
                assert not sn[e, :3].any() and sn[e, 3].any()
            else:
                assert np.array_equal(sn[e, :3], sp[e, 1:])
    assert n_done > 10


def test_observation_depends_on_the_action():
    a = rollout(4, 1, 1, p_done=0.0, action_seed=1)
    b = rollout(4, 1, 1, p_done=0.0, action_seed=2)
    assert not np.array_equal(a[1][3], b[1][3])          # the action streams differ
    assert not np.array_equal(a[1][0][:, 3], b[1][0][:, 3])
    assert np.array_equal(a[1][1], b[1][1])              # rewards come from the counters alone


def test_reward_and_termination_rates():
    tr = rollout(64, 8, 200, p_done=0.02, sprites=1)
    r = np.concatenate([t[1] for t in tr[1:]])
    d = np.concatenate([t[2] for t in tr[1:]])
    assert set(np.unique(r)) <= {-1.0, 0.0, 1.0}
    n = r.size
    assert abs((r == 1).mean() - 0.05) < 4 * np.sqrt(0.05 * 0.95 / n)
    assert abs((r == -1).mean() - 0.05) < 4 * np.sqrt(0.05 * 0.95 / n)
    assert abs(d.mean() - 0.02) < 4 * np.sqrt(0.02 * 0.98 / n)


def test_frames_are_sparse_with_bounded_sprites():
    s = rollout(3, 1, 0, sprites=10)[0][0]
    nz = (s[:, 3] != 0).sum(axis=(1, 2))
    assert (nz <= 10 * 64).all() and (nz >= 64).all()


def test_bad_arguments_are_rejected():
    L = A.lib()
    h = C.c_void_p()
    assert L.paac_actors_create(4, 1, 0, 0.1, 4, None) == -1
    for n_e, n_w, p, sp in [(0, 1, 0.1, 4), (4, 0, 0.1, 4), (4, 5, 0.1, 4), (4, 2, 1.5, 4), (4, 2, -0.1, 4), (4, 2, 0.1, -1)]:
        assert L.paac_actors_create(n_e, n_w, 0, p, sp, C.byref(h)) == -2
        assert not h.value
    assert L.paac_actors_reset(None, None) == -1
    assert L.paac_actors_create(4, 2, 0, 0.1, 4, C.byref(h)) == 0
    assert L.paac_actors_step(h, None, None, None, None) == -1
    L.paac_actors_destroy(h)
    L.paac_actors_destroy(None)
