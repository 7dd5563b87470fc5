#!/usr/bin/env python3
"""Benchmark of the VER learner step on one MI355X.

A "step" is one full PPO update over one synthetic ragged rollout held as the
linear collection buffer (steps in arrival order): ver_ingest and its gathers,
ver_gae and ver_is_weight once, then epochs x minibatches x (ver_pack_minibatch, ver_lstm_fwd,
ver_ppo_loss, ver_lstm_bwd, ver_adam_step).  All inputs are resident in HBM before the timed
region.  Prints ONE JSON line: learner env-steps/s, the roofline position of
the dominant kernel (timed with HIP events inside the library during the timed
region), the HBM-bound kernels on roofline-scale replicas of the workload, and
the CPU oracle timed on a bounded sample of the same workload.

    python bench.py [--workload max|large|manip|nav|tiny] [--steps K] [--warmup W]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}   # MI355X dense MFMA peaks
# One exchange of rows between the 32 workgroups of an XCD through its L2 (store, wait, flag, poll, load), measured
# on the box with a kernel that does nothing else: the least a timestep of the recurrence can cost in this design.
EXCHANGE_FLOOR_US = 1.0

MAX_IS = 1.0   # truncation of the importance weight (appendix hyper-parameter table)

TRAFFIC_PROFILE = os.path.join("profiles", "hbm_traffic_max_workload.md")


def traffic_from_profile(workload, kernel_symbol, root=ROOT):
    """HBM bytes per launch (read + written) of `kernel_symbol`, read from the committed summary of the rocprofv3
    FETCH_SIZE / WRITE_SIZE runs of this script (scaled there by a copy of known size).  The summary covers the
    `max` workload only; None for any other workload, or when the file or the kernel's row is missing."""
    if workload != "max":
        return None
    try:
        for line in open(os.path.join(root, TRAFFIC_PROFILE)):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) >= 7 and cells[1].startswith("`" + kernel_symbol):
                return (float(cells[5]) + float(cells[6])) * 1e6
    except (OSError, ValueError):
        pass
    return None


def collection_logp(ro, compute, x_bf16):
    """Log-probability the current weights give every stored action, evaluated
    over whole sequences on the GPU (input preparation, untimed), plus the
    workload's seeded noise: this is the rollout's logp_old."""
    import torch
    from paper_2210_05064_amd.learner import Learner
    w = ro["workload"]
    full = Learner(ro, compute=compute, x_bf16=x_bf16, minibatches=1)
    full.pack(0, 0)
    full.forward()
    torch.cuda.synchronize()
    u = full.head_out
    if w.dist == 0:
        logp = torch.log_softmax(u, dim=1).gather(1, full.act_packed.long().view(-1, 1)).squeeze(1)
    else:
        ls = full.log_std
        z = (full.act_packed - u) * torch.exp(-ls)
        logp = (-0.5 * z * z - ls - 0.5 * float(np.log(2 * np.pi))).sum(1)
    flat = torch.empty(ro["S"], device="cuda")
    flat[full.gather_idx.long()] = logp
    flat += torch.from_numpy(ro["logp_noise"]).cuda()
    torch.cuda.synchronize()
    del full
    torch.cuda.empty_cache()
    return flat


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(ro, budget_s=16.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload:
    bucketing, GAE and importance weights over the whole buffer, one minibatch's
    packing and loss in full, the Adam step over all weights, and the LSTM
    forward/backward over as many of that minibatch's pieces (shortest first) as
    fit the time budget, scaled to the whole update by step count.  The LSTM
    sample is timed twice, half the budget each: with the numerical library's
    thread pool limited to one thread, and with all threads it wants to use."""
    from oracle import (adam as oadam, gae as ogae, ingest as oing, is_weight as ois, lstm as olstm, pack as opack,
                        ppo_loss as oloss)
    from paper_2210_05064_amd import workloads as wl
    from threadpoolctl import threadpool_info, threadpool_limits
    w = ro["workload"]
    S, B, E = ro["S"], w.minibatches, w.epochs
    arr_env, arr_t, csr_of_arrival = wl.arrival_order(ro["env_off"], seed=1)
    t0 = time.perf_counter()
    _, order, _ = oing.ingest(arr_env, ro["N"], arr_t)
    for k in ("rewards", "values", "dones", "obs", "actions"):
        oing.to_env_major(ro[k][csr_of_arrival], order)
    t_ingest = time.perf_counter() - t0
    t0 = time.perf_counter()
    adv, ret = ogae.gae(ro["rewards"], ro["values"], ro["dones"], ro["last_values"], ro["env_off"], w.gamma, w.lam)
    is_w = ois.is_weights(ro["env_off"], MAX_IS)
    t_gae = time.perf_counter() - t0
    t0 = time.perf_counter()
    meta = opack.pack_minibatch(ro["dones"], ro["env_off"], ro["seq_key"][0], B, 0, ro["env_started_episode"])
    opack.gather_rows(ro["obs"], meta["gather_idx"])
    t_pack = time.perf_counter() - t0
    M = meta["M"]
    W = olstm.weights_f64(ro["weights"])
    rng = np.random.default_rng(0)

    def lstm_sample(budget):
        grads = olstm.zero_grads(W)
        steps = 0
        t0 = time.perf_counter()
        for j in range(meta["n_seq"] - 1, -1, -1):          # shortest pieces first
            f0, n = int(meta["seq_first"][j]), int(meta["seq_len"][j])
            u, v, saved = olstm.piece_forward(ro["obs"][f0:f0 + n], W)
            olstm.piece_backward(rng.standard_normal(u.shape) / M, rng.standard_normal(n) / M, W, saved, grads)
            steps += n
            if time.perf_counter() - t0 > budget:
                break
        return (time.perf_counter() - t0) * M / steps, steps

    with threadpool_limits(limits=1):
        t_lstm_1, steps_1 = lstm_sample(budget_s / 2)
    t_lstm, steps = lstm_sample(budget_s / 2)
    t0 = time.perf_counter()
    u = rng.standard_normal((M, w.act_dim))
    acts = opack.gather_rows(ro["actions"], meta["gather_idx"])
    oloss.ppo_loss(w.dist, u, rng.standard_normal(M), W["log_std"], acts, rng.standard_normal(M),
                   opack.gather_rows(adv, meta["gather_idx"]), opack.gather_rows(ret, meta["gather_idx"]),
                   w.clip, w.value_coef, w.entropy_coef, opack.gather_rows(is_w, meta["gather_idx"]))
    t_loss = time.perf_counter() - t0
    flat = [W["layers"][l][k] for l in range(w.n_layers) for k in ("W_ih", "W_hh", "b_ih", "b_hh")] + \
           [W["W_a"], W["b_a"], W["w_v"], W["b_v"], W["log_std"]]
    t0 = time.perf_counter()
    oadam.adam_step(flat, flat, [np.zeros_like(x) for x in flat], [np.zeros_like(x) for x in flat], 1, 2.5e-4)
    t_adam = time.perf_counter() - t0
    rest = t_ingest + t_gae + E * B * (t_pack + t_loss + t_adam)   # plain Python / numpy loops: one thread
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return {
        "value": S / (rest + E * B * t_lstm), "unit": "env-steps/s", "cores": int(threads), "kind": "oracle",
        "value_single_thread": S / (rest + E * B * t_lstm_1),
        "cpu_model": _cpu_model(), "logical_cpus": os.cpu_count(), "usable_cpus": usable,
        "implementation": "oracle/ as it stands: numpy fp64, Python loops per environment / piece / row; only its "
                          "matrix-vector products (numpy's BLAS) use more than one thread",
        "sample": (f"bucketing of the arrival-order buffer ({t_ingest:.2f}s); GAE and importance weights on all {S} steps "
                   f"({t_gae:.2f}s); packing ({t_pack:.2f}s) and loss ({t_loss:.2f}s) of one minibatch of {M} rows in full; "
                   f"LSTM fwd+bwd on that minibatch's shortest pieces, scaled to {M} rows: {steps_1} steps with one thread "
                   f"({t_lstm_1:.1f}s per minibatch), {steps} steps with {threads} threads ({t_lstm:.1f}s per minibatch); "
                   f"Adam step on all weights ({t_adam:.2f}s); update = bucketing + GAE + {E}x{B} minibatches"),
    }


LSTM_CLASSES = ("lstm_prep", "lstm_gemm_fwd", "lstm_rec_fwd", "lstm_rec_bwd", "lstm_gemm_dx", "lstm_gemm_dw", "lstm_dbias")
SCALAR_NAMES = ["total", "policy", "value", "entropy", "approx_kl", "clip_frac"]


def measure(workload, seed, steps, warmup, env_major, headline):
    """`warmup` untimed and `steps` timed PPO updates of one workload, then one more update with every kernel class
    bracketed by events.  Returns (result dict, rollout).  headline: the full JSON line of the run's main workload;
    otherwise the short record that goes into `other_workloads`."""
    import torch
    from paper_2210_05064_amd import binding as ver, workloads as wl
    from paper_2210_05064_amd.learner import Learner
    w = wl.WORKLOADS[workload]
    ro = wl.make_rollout(w, seed=seed)
    # the loss carries VER's truncated importance weight, and the optimiser runs inside the update: Adam with the
    # paper's cosine schedule over its 500 M training steps
    learner = Learner(ro, adam_total_steps=max(1, int(500e6 // ro["S"])) * w.epochs * w.minibatches, max_is=MAX_IS,
                      arrival=None if env_major else wl.arrival_order(ro["env_off"], seed=seed + 1))
    learner.set_logp_old(collection_logp(ro, learner.compute, learner.x_bf16))
    torch.cuda.synchronize()

    # the loss scalars of every minibatch of the FIRST update ever run on these weights (a warm-up update unless
    # warmup = 0), copied device to device without synchronising: the later updates reuse the same rollout with
    # the optimiser on, so their scalars describe a policy that has moved away from the one that collected it
    n_mb = w.epochs * learner.B
    first_scalars = torch.zeros((n_mb, 6), dtype=torch.float32, device="cuda")
    log_first = lambda e, b: first_scalars[e * learner.B + b].copy_(learner.scalars)
    first = True
    for _ in range(warmup):
        learner.update(on_minibatch=log_first if first else None)
        first = False
    torch.cuda.synchronize()
    if learner.lstm_timed_out() or learner.gae_timed_out():
        print("device-side wait timed out during warm-up", file=sys.stderr)
        sys.exit(4)

    rec_mask = (1 << ver.PROF_CLASSES.index("lstm_rec_fwd")) | (1 << ver.PROF_CLASSES.index("lstm_rec_bwd"))
    ver.ver_profile_enable(rec_mask)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        learner.update(on_minibatch=log_first if first else None)
        first = False
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = ver.ver_profile_read()
    ver.ver_profile_enable(0)
    if learner.lstm_timed_out() or learner.gae_timed_out():
        print("device-side wait timed out during the timed region: results are invalid", file=sys.stderr)
        sys.exit(4)
    scalars = learner.scalars.cpu().numpy().tolist()
    first_scalars = first_scalars.cpu().numpy()
    # T_max and pieces of every minibatch of an update (the same in every update: same rollout, same keys)
    t_maxes = sorted(int(ix["info"][1].item()) for ix in learner.index_sets)
    n_seqs = sorted(int(ix["info"][0].item()) for ix in learner.index_sets)

    # every kernel class once more, for the breakdown (untimed)
    ver.ver_profile_enable((1 << len(ver.PROF_CLASSES)) - 1)
    learner.update()
    torch.cuda.synchronize()
    full = ver.ver_profile_read()
    ver.ver_profile_enable(0)

    S, M, H = learner.S, learner.M, w.hidden
    ms_per_step = 1e3 * elapsed / steps
    dom = max(("lstm_rec_fwd", "lstm_rec_bwd"), key=lambda k: prof[k][0])
    dom_ms, dom_n = prof[dom]
    # recurrent product of one layer over all timesteps of a minibatch: 2 * (4H x H) * rows.  With two layers one
    # launch runs both time loops and the projection between them (the same number of FLOPs again).
    flops_per_launch = 8.0 * H * H * M * (3 if w.n_layers == 2 else 1)
    achieved = flops_per_launch / (dom_ms / dom_n * 1e-3) / 1e12
    dtype = "bf16" if learner.compute else "f32"
    symbol = ("lstm_pipe_" if w.n_layers == 2 else "lstm_rec_") + dom[-3:] + "_kernel"
    # the whole LSTM: forward contractions 2 * 4H * (D_l + H) per row and layer, backward twice that (data and
    # weight gradients); time = every LSTM kernel class of one update (weight preparation, input projections, time
    # loops, weight and bias gradients), from the breakdown update
    fwd_flops_row = sum(2.0 * 4 * H * ((w.input_dim if l == 0 else H) + H) for l in range(w.n_layers))
    lstm_flops = 3.0 * fwd_flops_row * S * w.epochs
    lstm_ms = sum(full[k][0] for k in LSTM_CLASSES)
    lstm_total = lstm_flops / (lstm_ms * 1e-3) / 1e12
    # what the chain of dependent timesteps allows: every minibatch runs T_max steps forward and T_max backward, each
    # at least one exchange between the workgroups that share the hidden units (EXCHANGE_FLOOR_US, measured)
    chain_ms = sum(t_maxes) * 2 * EXCHANGE_FLOOR_US * 1e-3
    roofline = {"bound": "mfma", "kernel": dom, "kernel_symbol": symbol,
                "achieved": achieved, "peak": PEAK_TFLOPS[dtype],
                "unit": "TFLOP/s", "frac": achieved / PEAK_TFLOPS[dtype],
                "traffic": traffic_from_profile(w.name, symbol), "traffic_source": TRAFFIC_PROFILE if w.name == "max" else None,
                "avg_launch_ms": dom_ms / dom_n, "launches": dom_n, "flops_per_launch": flops_per_launch,
                "T_max_min_median_max": [t_maxes[0], t_maxes[len(t_maxes) // 2], t_maxes[-1]],
                "pieces_min_median_max": [n_seqs[0], n_seqs[len(n_seqs) // 2], n_seqs[-1]],
                "lstm_total": {"flops_per_update": lstm_flops, "ms_per_update": lstm_ms, "achieved": lstm_total,
                               "frac": lstm_total / PEAK_TFLOPS[dtype], "classes": list(LSTM_CLASSES)},
                "latency_bound": {"exchange_floor_us": EXCHANGE_FLOOR_US, "dependent_steps_per_update": 2 * sum(t_maxes),
                                  "floor_ms_per_update": chain_ms,
                                  "time_loops_ms_per_update": full["lstm_rec_fwd"][0] + full["lstm_rec_bwd"][0],
                                  "achieved_over_attainable": chain_ms / (full["lstm_rec_fwd"][0] + full["lstm_rec_bwd"][0])}}
    if not headline:
        return {"workload": w.name, "dtype": dtype, "value": S / (elapsed / steps), "unit": "env-steps/s",
                "ms_per_step": ms_per_step, "steps": steps, "warmup": warmup,
                "rollout_steps": S, "rows_per_minibatch": M, "lstm": f"{w.n_layers}x{w.hidden}",
                "dominant_kernel": symbol, "frac": roofline["frac"], "lstm_total_frac": roofline["lstm_total"]["frac"],
                "T_max_min_median_max": roofline["T_max_min_median_max"],
                "time_loops_ms_per_update": roofline["latency_bound"]["time_loops_ms_per_update"],
                "clip_frac_first_update": float(first_scalars[:, 5].mean())}, ro
    out = {
        "metric": "learner env-steps/sec per PPO update (1 MI355X)",
        "value": S / (elapsed / steps), "unit": "env-steps/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": w.name, "n_envs": w.n_envs, "rollout_steps": S, "input_dim": w.input_dim,
                   "lstm": f"{w.n_layers}x{w.hidden}", "policy": "categorical" if w.dist == 0 else "gaussian",
                   "act_dim": w.act_dim, "epochs": w.epochs, "minibatches": w.minibatches,
                   "rows_per_minibatch": M, "seed": seed},
        "step_passes_per_sec": S * w.epochs / (elapsed / steps),
        "roofline": roofline,
        "kernel_ms_per_update": {k: round(v[0], 4) for k, v in full.items()},
        "kernel_launches_per_update": {k: v[1] for k, v in full.items()},
        "loss_scalars_first_update": {"first_minibatch": dict(zip(SCALAR_NAMES, first_scalars[0].tolist())),
                                      "last_minibatch": dict(zip(SCALAR_NAMES, first_scalars[-1].tolist()))},
        "loss_scalars_last_minibatch": dict(zip(SCALAR_NAMES, scalars)),
    }
    del learner
    return out, ro


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="max")
    ap.add_argument("--seed", type=int, default=4000)
    ap.add_argument("--cpu-budget", type=float, default=15.0, help="seconds of oracle LSTM work (0 = skip)")
    ap.add_argument("--env-major", action="store_true",
                    help="hand the rollout over already bucketed by environment (skips ver_ingest)")
    ap.add_argument("--no-replica", action="store_true",
                    help="leave the roofline-scale replicas of the HBM-bound kernels out of the JSON line")
    ap.add_argument("--no-others", action="store_true",
                    help="leave the short runs of the other workloads (nav, manip, large, tiny) out of the JSON line")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="only run three device-to-device copies of MIB mebibytes (a kernel of known HBM traffic "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters by) and exit")
    ap.add_argument("--hbm-replica", nargs="?", const="all", default=None, metavar="SECTIONS",
                    help="instead of the update, run every HBM-bound kernel on a roofline-scale replica of the max "
                         "workload (gigabytes per launch) and print bytes / time against the HBM peak as one JSON line; "
                         "optionally a comma-separated subset of gae,pack,loss,adam,ingest")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the learner step of ONE GPU; runs on several GPUs are not part of this build "
              "(the path would shard by data parallelism with one gradient all-reduce per minibatch)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2210_05064_amd import binding as ver, workloads as wl
    from paper_2210_05064_amd.learner import Learner
    if not torch.cuda.is_available():
        print("no GPU visible: the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)

    if args.copy_calibration > 0:
        src = torch.ones(args.copy_calibration << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": src.numel() * 4, "copy_calibration_bytes_written": src.numel() * 4}))
        return

    if args.hbm_replica:
        from paper_2210_05064_amd import hbm_replica
        only = None if args.hbm_replica == "all" else args.hbm_replica.split(",")
        print(json.dumps({"hbm_replica": hbm_replica.run(seed=args.seed + 3000, reps=max(1, args.steps) * 2, only=only)}))
        return

    out, ro = measure(args.workload, args.seed, args.steps, args.warmup, args.env_major, headline=True)
    if not args.no_others:
        # the paper-shaped smaller workloads (navigation, manipulation, the larger per-GPU batch and the tiny case),
        # a few updates each, measured the same way
        out["other_workloads"] = []
        for k, name in enumerate(n for n in ("nav", "manip", "large", "tiny") if n != args.workload):
            o, _ = measure(name, args.seed + 10 * (k + 1), steps=10, warmup=3, env_major=args.env_major, headline=False)
            out["other_workloads"].append(o)
    if not args.no_replica:
        # the HBM-bound kernels once more on gigabyte-sized replicas of the workload (untimed part of the run): at the
        # workload's own sizes they sit at the launch-latency floor, which says nothing about the kernels
        torch.cuda.empty_cache()
        try:
            from paper_2210_05064_amd import hbm_replica
            out["hbm_replica"] = [{k: r[k] for k in ("kernel", "shape", "bytes", "ms", "achieved", "peak", "unit", "frac")}
                                  for r in hbm_replica.run(seed=args.seed + 3000, reps=20)]
        except Exception as e:   # the headline figures above do not depend on this part
            out["hbm_replica_error"] = repr(e)
    if args.cpu_budget > 0:
        out["cpu_baseline"] = cpu_baseline(ro, args.cpu_budget)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
