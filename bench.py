#!/usr/bin/env python3
"""Benchmark of the PAAC hot path on one MI355X.

One "step" is one PAAC iteration without the environments (Algorithm 1, the body of the repeat
loop): t_max calls of paac_select_actions, one per timestep slab, followed by one
paac_train_step over the n_e x t_max rollout.  Inputs are synthetic, seeded, and resident in HBM
before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 0..4] [--n_e N] [--t_max T] [--no-cpu-baseline]
                    [--phase both|select|train]

--phase select / train runs only that call in every loop of the run (for profiler runs whose rows
must not mix the two calls' launches of one kernel); the reported value is then not the metric.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X dense fp32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0    # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0

# Kernels of the fp32 configuration that issue bf16 MFMAs on exact operand parts (bytes are exact in
# bf16; an fp32 number is the sum of three bf16 parts): name -> bf16 multiply-accumulates issued per
# algorithmic fp32 one.  Their rate is reported against the fp32 matrix peak as algorithmic work and,
# times this factor, against the bf16 matrix peak as issued work.
def bf16_parts_per_mac(name, rows):
    """rows: states in the launch.  The first layer (forward, weight gradient) always runs on exact
    parts (bytes x three weight / gradient parts); layers 2-3 forward from 96 states per launch on (six
    part products per multiply-accumulate), alone or with the first layer in one launch."""
    if name.endswith("conv1_fwd") or name.endswith("conv1_wgrad"):
        return 3.0
    if name.endswith("convs_fwd"):
        return 5.3            # FLOP-weighted mean of 3 (first layer) and 6 (layers 2-3) on the Nature network
    if rows >= 96 and (name.endswith("conv2_fwd") or name.endswith("conv3_fwd")):
        return 6.0
    return 0.0


def kernel_work(net, n_e, t_max, act_bytes=4):
    """Algorithmic work per launch of every kernel: ('flop', 2 x MACs) or ('byte', HBM bytes)."""
    B, Bp, A = n_e * t_max, n_e * (t_max + 1), net.n_actions
    shapes = net.conv_out_shapes()
    cin = net.in_c
    conv = []
    for (co, k, s), (c, h, w) in zip(net.conv, shapes):
        conv.append(2.0 * h * w * (k * k * cin) * co)
        cin = co
    fc = 2.0 * net.flat() * net.fc
    hd = 2.0 * net.fc * (A + 1)
    P = net.param_count()
    w = {}
    for l, f in enumerate(conv):
        w[f"select.conv{l + 1}_fwd"] = ("flop", f * n_e)
        w[f"train.conv{l + 1}_fwd"] = ("flop", f * Bp)
        w[f"train.conv{l + 1}_wgrad"] = ("flop", f * B)
        if l > 0:
            w[f"train.conv{l + 1}_dgrad"] = ("flop", f * B)
    w["select.convs_fwd"] = ("flop", sum(conv) * n_e)    # all convolutions of a sample in one workgroup
    w["train.convs_fwd"] = ("flop", sum(conv) * Bp)
    w["select.fc_fwd"] = ("flop", fc * n_e)
    w["train.fc_fwd"] = ("flop", fc * Bp)
    w["train.fc_wgrad"] = ("flop", fc * B)
    w["train.fc_dgrad"] = ("flop", fc * B)
    w["train.fc_bwd"] = ("flop", 2 * fc * B)
    for l in range(1, len(conv)):
        w[f"train.conv{l + 1}_bwd"] = ("flop", 2 * conv[l] * B)
    # algorithmic HBM bytes of the first-layer forward pass per state (the bound of that kernel in the
    # bf16 configuration): the uint8 state in, the activations out (2 bytes each in bf16, else 4)
    c1 = shapes[0]
    w["_conv1_fwd_bytes_per_state"] = ("byte", float(net.in_c * net.in_h * net.in_w + act_bytes * c1[0] * c1[1] * c1[2]))
    w["select.heads_sample"] = ("flop", hd * n_e)
    w["train.heads_fwd"] = ("flop", hd * Bp)
    w["train.heads_bwd"] = ("flop", 2 * hd * B)
    w["train.returns_loss"] = ("byte", 4.0 * (Bp * (A + 1) + B * (A + 4)))
    w["train.grad_reduce_norm"] = ("byte", 8.0 * P)      # read one gradient copy, write the arena
    w["train.clip_rmsprop"] = ("byte", 20.0 * P)         # read theta, g, g2; write theta, g2
    w["train.bf16_weight_copies"] = ("byte", 8.0 * P)    # read the fp32 weights, write two bf16 copies
    return w


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=2, help="index into the measurement configurations")
    ap.add_argument("--rollouts", type=int, default=4, help="distinct resident rollouts rotated through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-steps", type=int, default=50)
    ap.add_argument("--phase", choices=["both", "select", "train"], default="both",
                    help="run only this call in every loop (profiler runs); 'both' is the metric")
    ap.add_argument("--n_e", type=int, default=0, help="override the configuration's environment count (n_e sweep)")
    ap.add_argument("--t_max", type=int, default=0, help="override the configuration's rollout length")
    ap.add_argument("--lr", type=float, default=0.0, help="override the configuration's learning rate")
    ap.add_argument("--algorithm", choices=["a2c", "nstep-q"], default="a2c",
                    help="a2c: the paper's actor-critic (the reported metric); nstep-q: the value-based variant on the same kernels")
    ap.add_argument("--epsilon", type=float, default=0.1, help="exploration rate of --algorithm nstep-q")
    ap.add_argument("--sweep-ne", default="", help="comma separated n_e values: one line with the throughput at each (lr = 0.0007 n_e)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import numpy as np
    import torch
    from paper_1705_04862_amd import inputs as I
    from paper_1705_04862_amd import paac as P

    import dataclasses
    cfg = I.CONFIGS[args.config]
    if args.sweep_ne:
        # the paper's n_e study: the same network at several n_e with lr = 0.0007 n_e (throughput only)
        rows = []
        for ne in [int(x) for x in args.sweep_ne.split(",")]:
            sub = [sys.executable, os.path.abspath(__file__), "--config", str(args.config), "--n_e", str(ne), "--lr", repr(0.0007 * ne),
                   "--steps", str(args.steps), "--warmup", str(args.warmup), "--no-cpu-baseline", "--profile-steps", "5"]
            import subprocess
            line = subprocess.run(sub, check=True, capture_output=True, text=True).stdout.strip().splitlines()[-1]
            d = json.loads(line)
            rows.append({"n_e": ne, "lr": 0.0007 * ne, "value": d["value"], "ms_per_step": d["ms_per_step"],
                         "pct_mfma_peak_whole_step": d["pct_mfma_peak_whole_step"], "launch": d["config"]["launch"]})
        print(json.dumps({"metric": "env-timesteps/sec (select+train) over n_e, lr = 0.0007 n_e", "unit": "env-timesteps/s",
                          "n_gpus": 1, "data": "synthetic", "config": {"workload": cfg.name + " with n_e swept", "t_max": cfg.t_max},
                          "sweep": rows}))
        return
    if args.n_e or args.t_max or args.lr:
        cfg = dataclasses.replace(cfg, n_e=args.n_e or cfg.n_e, t_max=args.t_max or cfg.t_max,
                                  hp=dataclasses.replace(cfg.hp, lr=args.lr or cfg.hp.lr))
    net, n_e, T = cfg.net, cfg.n_e, cfg.t_max
    torch.cuda.set_device(0)
    ctx = P.Paac(net.arch, n_e, T, net.n_actions, cfg.precision)
    params = I.config_params(cfg)
    ctx.set_state(params)
    if args.algorithm == "nstep-q":
        ctx.set_algorithm(P.PAAC_ALG_NSTEP_Q, args.epsilon)

    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    host_rollouts = [I.config_rollout(cfg, k) for k in range(args.rollouts)]
    R = []
    for ro in host_rollouts:
        R.append(dict(states=to_dev(ro.states), rewards=to_dev(ro.rewards), dones=to_dev(ro.dones),
                      uniforms=to_dev(ro.uniforms),
                      actions=torch.zeros(T, n_e, dtype=torch.int32, device="cuda:0"),
                      values=torch.zeros(T, n_e, dtype=torch.float32, device="cuda:0")))
    stats = torch.zeros(8, dtype=torch.float32, device="cuda:0")

    def step(i, what=None):
        what = what or args.phase
        r = R[i % len(R)]
        if what in ("both", "select"):
            for t in range(T):
                ctx.select_actions(r["states"][t], r["uniforms"][t], r["actions"][t], r["values"][t])
        if what in ("both", "train"):
            ctx.train_step(r["states"], r["actions"], r["rewards"], r["dones"], cfg.hp, stats)

    def timed(k, what=None):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(k):
            step(i, what)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    # Launch mode: the library can replay captured HIP graphs (one per call) or launch its kernels one
    # by one.  Which is faster depends on the host (a graph launch has a fixed cost per call, direct
    # launches need a host that keeps ahead of the GPU): a short calibration picks the mode, the timed
    # region then runs entirely in that mode.
    for i in range(args.warmup):
        step(i)
    k2 = max(10, args.steps // 10)
    ms_graph = 1e3 * timed(k2) / k2
    ctx.set_graphs(False)
    for i in range(5):
        step(i)
    ms_eager = 1e3 * timed(k2) / k2
    use_graphs = ms_graph <= ms_eager
    ctx.set_graphs(use_graphs)
    for i in range(5):
        step(i)
    elapsed = timed(args.steps)
    ms_per_step = 1e3 * elapsed / args.steps
    value = args.steps * n_e * T / elapsed

    # context figures: the halves of the step
    ms_select = 1e3 * timed(k2, "select") / k2 if args.phase != "train" else 0.0
    ms_train = 1e3 * timed(k2, "train") / k2 if args.phase != "select" else 0.0
    # context: the same step with the opt-in rollout activation cache (the train step reuses the
    # activations of the t_max select calls and only runs the forward pass of the bootstrap states);
    # never the reported value
    ctx.set_activation_cache(True)
    for i in range(5):
        step(i)
    ms_cached = 1e3 * timed(k2) / k2
    ctx.set_activation_cache(False)

    per_kernel, roof = {}, None
    bf16cfg = cfg.precision == 1
    mfma_peak = PEAK_BF16_MFMA_TFLOPS if bf16cfg else PEAK_FP32_MFMA_TFLOPS
    if args.profile_steps > 0:
        # per-kernel durations with HIP events on the library's stream
        ctx.set_profiling(True)
        for i in range(args.profile_steps):
            step(i)
        times = ctx.kernel_times()
        ctx.set_profiling(False)
        work = kernel_work(net, n_e, T, 2 if cfg.precision == 1 else 4)
        per_kernel = {}
        for name, t in times.items():
            avg_us = 1e3 * t["ms"] / t["calls"]
            kind, amount = work[name]
            per_kernel[name] = dict(avg_us=round(avg_us, 3), calls_per_step=t["calls"] / args.profile_steps,
                                    us_per_step=round(1e3 * t["ms"] / args.profile_steps, 3))
            if kind == "flop":
                per_kernel[name]["tflops"] = round(amount / (avg_us * 1e-6) / 1e12, 3)
            else:
                per_kernel[name]["gbs"] = round(amount / (avg_us * 1e-6) / 1e9, 1)
        bf16cfg = cfg.precision == 1
        mfma_peak = PEAK_BF16_MFMA_TFLOPS if bf16cfg else PEAK_FP32_MFMA_TFLOPS
        for name, k in per_kernel.items():
            if "tflops" in k:
                k["frac_of_peak"] = round(k["tflops"] / mfma_peak, 4)
                parts = 0.0 if bf16cfg else bf16_parts_per_mac(name, n_e if name.startswith("select.") else n_e * (T + 1))
                if parts:                                              # issued bf16 work against the bf16 peak
                    k["bf16_parts_per_mac"] = parts
                    k["frac_of_bf16_peak_issued"] = round(k["tflops"] * parts / PEAK_BF16_MFMA_TFLOPS, 4)
            else:
                k["frac_of_peak"] = round(k["gbs"] / PEAK_HBM_GBS, 4)
        dom = max(per_kernel, key=lambda n: per_kernel[n]["us_per_step"])
        kind, amount = work[dom]
        traffic = None
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
        if os.path.exists(tpath) and not (args.n_e or args.t_max):      # counters were taken at the configuration's own size
            traffic = json.load(open(tpath)).get(f"cfg{args.config}", {}).get(dom)
        avg_s = per_kernel[dom]["avg_us"] * 1e-6
        # Which roof bounds the dominant kernel is decided by the evidence: its algorithmic FLOP rate as a
        # fraction of the matrix peak against its algorithmic HBM byte rate as a fraction of 8 TB/s (for a
        # contraction without a stated byte figure, the counter-measured bytes per launch where the counters
        # were taken at this size); the larger fraction names the roof the kernel is closer to.
        states = n_e if dom.startswith("select.") else n_e * (T + 1)
        alg_bytes = work["_conv1_fwd_bytes_per_state"][1] * states if dom.endswith("conv1_fwd") else None
        mfma_frac = amount / avg_s / 1e12 / mfma_peak if kind == "flop" else 0.0
        hbm_bytes = amount if kind == "byte" else (alg_bytes if alg_bytes else traffic)
        hbm_frac = hbm_bytes / avg_s / 1e9 / PEAK_HBM_GBS if hbm_bytes else 0.0
        if kind == "flop" and mfma_frac >= hbm_frac:
            roof = dict(bound="mfma", kernel=dom, achieved=round(amount / avg_s / 1e12, 3), peak=mfma_peak, unit="TFLOP/s",
                        frac=round(mfma_frac, 4), traffic=traffic, avg_launch_us=per_kernel[dom]["avg_us"],
                        algorithmic_flop_per_launch=amount, hbm_frac_of_same_kernel=round(hbm_frac, 4))
        else:
            ab = amount if kind == "byte" else (alg_bytes if alg_bytes else hbm_bytes)
            roof = dict(bound="hbm", kernel=dom, achieved=round(ab / avg_s / 1e9, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(ab / avg_s / 1e9 / PEAK_HBM_GBS, 4), traffic=traffic, avg_launch_us=per_kernel[dom]["avg_us"],
                        algorithmic_bytes_per_launch=ab, mfma_frac_of_same_kernel=round(mfma_frac, 4))
        if "bf16_parts_per_mac" in per_kernel[dom]:
            roof["note"] = ("this kernel issues %.1f bf16 MFMA multiply-accumulates per algorithmic fp32 one (exact operand parts): "
                            "%.4f of the bf16 matrix peak as issued work" % (per_kernel[dom]["bf16_parts_per_mac"], per_kernel[dom]["frac_of_bf16_peak_issued"]))


    sel_f, trn_f = ctx.flops()
    step_flop = T * sel_f + trn_f
    out = {
        "metric": "env-timesteps/sec (select+train) at n_e=%d,t_max=%d; %% MFMA peak" % (n_e, T) +
                  ("" if args.algorithm == "a2c" else " [value-based variant, not the paper's measured method]"),
        "value": round(value, 1), "unit": "env-timesteps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.precision == 1 else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "net": net.name, "n_e": n_e, "t_max": T, "n_actions": net.n_actions,
                   "rollouts_rotated": len(R), "algorithm": args.algorithm, "phase": args.phase,
                   "launch": "hip-graph replay (t_max select graphs + 1 train graph)" if use_graphs else "direct kernel launches on one stream"},
        "roofline": roof,
        "step_gflop": round(step_flop / 1e9, 3),
        "pct_mfma_peak_whole_step": round(100 * step_flop / elapsed * args.steps / (mfma_peak * 1e12), 3),
        "ms_select_x_tmax": round(ms_select, 4), "ms_train": round(ms_train, 4),
        "ms_per_step_graph_replay": round(ms_graph, 4), "ms_per_step_direct_launch": round(ms_eager, 4),
        "ms_per_step_with_activation_cache": round(ms_cached, 4),
        "kernels": per_kernel,
        "paper_context": "derived from the paper's Table 1 training times and time split on a GTX 980 Ti: "
                         "about 7200 (arch_nips) / 4100-4300 (arch_nature) env-timesteps/s for this path",
    }

    if not args.no_cpu_baseline and args.phase == "both":
        from oracle import paac_oracle as O
        ro = host_rollouts[0]
        rms = I.make_rms(0, net)

        def oracle_iter():
            if args.algorithm == "nstep-q":
                for t in range(T):
                    O.q_select_actions(net, params, ro.states[t], ro.uniforms[t], args.epsilon)
                O.q_train_step(net, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, cfg.hp)
                return
            for t in range(T):
                O.select_actions(net, params, ro.states[t], ro.uniforms[t])
            O.train_step(net, params, rms, ro.states, ro.actions, ro.rewards, ro.dones, cfg.hp)
        t0 = time.perf_counter()
        oracle_iter()
        first = time.perf_counter() - t0
        if first >= 5.0:                      # one iteration is already a bounded sample (the large configurations)
            reps, el = 1, first
        else:
            reps = int(max(1, min(20, 10.0 / max(first, 1e-3))))
            t0 = time.perf_counter()
            for _ in range(reps):
                oracle_iter()
            el = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(reps * n_e * T / el, 2), "unit": "env-timesteps/s",
                               "cores": O.threads(), "kind": "oracle",
                               "sample": "%d full iterations (t_max selects + 1 train) of %s" % (reps, cfg.name)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
