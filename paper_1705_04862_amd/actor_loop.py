"""Algorithm 1 end to end on one GPU with the synthetic environment: n_w host workers step n_e
environments, the master uploads the batched states, samples the actions on the GPU, and every
t_max steps runs the update (paper Section 3 "Parallel Framework").

    python -m paper_1705_04862_amd.actor_loop --config 2 --workers 8 --iters 200

Prints one JSON line: whole-loop timesteps per second (no synchronisation beyond what the algorithm
needs: the actions must reach the host before the environments can step) and, from a second pass
that synchronises after every phase, where the time of one iteration goes (environment, upload,
action selection incl. the copy of the actions to the host, update).  The paper reports the same
split for its CPU emulators (Section 5: 22 % / 50 % of the time in the emulator for the two nets).
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import time

import torch

from . import actors as A
from . import inputs as I
from . import paac as P


def run(cfg: I.Config, n_w: int, iters: int, warmup: int, sprites: int, seed: int, cache: bool, split: bool,
        graphs: bool = False, record: dict | None = None):
    """record: if a dict, the last iteration's inputs and results are copied into it (parameters and
    RMSProp state before the update, the rollout, the uniforms, then state, gradient and statistics
    after the update) so that a caller can replay that iteration elsewhere."""
    dev = torch.device("cuda:0")
    n_e, t_max, net = cfg.n_e, cfg.t_max, cfg.net
    stream = torch.cuda.Stream(device=dev)
    ctx = P.Paac(net.arch, n_e, t_max, net.n_actions, cfg.precision, stream=stream)
    ctx.init_params(seed)
    ctx.set_activation_cache(cache)
    ctx.set_graphs(graphs)
    env = A.Actors(n_e, n_w, seed=seed, p_done=cfg.p_done, sprites=sprites)

    obs = (4, 84, 84)
    states_h = torch.empty((n_e,) + obs, dtype=torch.uint8, pin_memory=True)
    actions_h = torch.empty(n_e, dtype=torch.int32, pin_memory=True)
    rewards_h = torch.empty((t_max, n_e), dtype=torch.float32, pin_memory=True)
    dones_h = torch.empty((t_max, n_e), dtype=torch.uint8, pin_memory=True)
    s_np, a_np, r_np, d_np = states_h.numpy(), actions_h.numpy(), rewards_h.numpy(), dones_h.numpy()
    states_d = torch.empty((t_max + 1, n_e) + obs, dtype=torch.uint8, device=dev)
    actions_d = torch.empty((t_max, n_e), dtype=torch.int32, device=dev)
    rewards_d = torch.empty((t_max, n_e), dtype=torch.float32, device=dev)
    dones_d = torch.empty((t_max, n_e), dtype=torch.uint8, device=dev)
    uniforms_d = torch.empty((t_max, n_e), dtype=torch.float32, device=dev)
    stats_d = torch.zeros(8, dtype=torch.float32, device=dev)

    env.reset(s_np)
    phase = {"env": 0.0, "upload": 0.0, "select": 0.0, "train": 0.0}

    def mark(name, t0):
        if split:
            stream.synchronize()
            phase[name] += time.perf_counter() - t0

    with torch.cuda.stream(stream):
        states_d[0].copy_(states_h, non_blocking=True)
        stream.synchronize()
        t_start = None
        for it in range(warmup + iters):
            if it == warmup:
                stream.synchronize()
                for k in phase:
                    phase[k] = 0.0
                t_start = time.perf_counter()
            ctx.fill_uniforms(seed, it * t_max * n_e, uniforms_d)
            for t in range(t_max):
                t0 = time.perf_counter()
                ctx.select_actions(states_d[t], uniforms_d[t], actions_d[t])
                actions_h.copy_(actions_d[t], non_blocking=True)
                stream.synchronize()                      # the workers need the actions
                if split:
                    phase["select"] += time.perf_counter() - t0
                t0 = time.perf_counter()
                env.step(a_np, s_np, r_np[t], d_np[t])
                if split:
                    phase["env"] += time.perf_counter() - t0
                t0 = time.perf_counter()
                states_d[t + 1].copy_(states_h, non_blocking=True)
                # the next environment step overwrites states_h: the copy has to be complete by
                # then, which the synchronisation after the next select guarantees (same stream)
                mark("upload", t0)
            t0 = time.perf_counter()
            rewards_d.copy_(rewards_h, non_blocking=True)
            dones_d.copy_(dones_h, non_blocking=True)
            last = record is not None and it == warmup + iters - 1
            if last:
                stream.synchronize()
                record["params"], record["rms"], _ = ctx.get_state(want_grads=False)
                for name, tns in (("states", states_d), ("actions", actions_d), ("rewards", rewards_d),
                                  ("dones", dones_d), ("uniforms", uniforms_d)):
                    record[name] = tns.cpu().numpy().copy()
            ctx.train_step(states_d, actions_d, rewards_d, dones_d, cfg.hp, stats_d)
            if last:
                stream.synchronize()
                record["params_after"], record["rms_after"], record["grads"] = ctx.get_state()
                record["outputs"] = ctx.get_train_outputs()
            states_d[0].copy_(states_d[t_max], non_blocking=True)
            mark("train", t0)
        stream.synchronize()
        wall = time.perf_counter() - t_start
    stats = ctx.read_stats(stats_d)
    env.close()
    ctx.close()
    return wall, phase, stats


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--workers", type=int, default=8)
    ap.add_argument("--iters", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--sprites", type=int, default=24)
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--n-e", type=int, default=0)
    ap.add_argument("--cache", type=int, default=1)
    args = ap.parse_args()
    cfg = I.CONFIGS[args.config]
    if args.n_e:
        cfg = dataclasses.replace(cfg, n_e=args.n_e)
    n_w = min(args.workers, cfg.n_e)
    wall_s, phase, _ = run(cfg, n_w, args.iters, args.warmup, args.sprites, args.seed, bool(args.cache), True)
    wall, _, stats = run(cfg, n_w, args.iters, args.warmup, args.sprites, args.seed, bool(args.cache), False)
    steps = args.iters * cfg.t_max * cfg.n_e
    tot = sum(phase.values())
    print(json.dumps({
        "metric": "actor_loop_timesteps_per_second", "value": steps / wall, "unit": "env-steps/s",
        "config": {"workload": cfg.name, "workers": n_w, "environment": f"synthetic, {args.sprites} sprites/frame",
                   "activation_cache": bool(args.cache)},
        "iters": args.iters, "ms_per_iteration": 1e3 * wall / args.iters,
        "split_ms_per_iteration": {k: 1e3 * v / args.iters for k, v in phase.items()},
        "split_fraction": {k: v / tot for k, v in phase.items()},
        "ms_per_iteration_synchronised": 1e3 * wall_s / args.iters,
        "last_stats": stats,
    }))


if __name__ == "__main__":
    main()
