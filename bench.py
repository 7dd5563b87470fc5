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

# HBM bytes per launch (read + written) of the dominant kernel class (with two layers: the launch that runs both
# time loops of one direction), from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this script, scaled by a copy of
# known size: see profiles/hbm_traffic_max_workload.md.  None where unmeasured.
MAX_IS = 1.0   # truncation of the importance weight (appendix hyper-parameter table)

MEASURED_TRAFFIC = {("max", "lstm_rec_bwd"): 1786.0e6, ("max", "lstm_rec_fwd"): 2004.5e6}


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


def cpu_baseline(ro, budget_s=15.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload:
    GAE over the whole buffer, one minibatch's packing and loss in full, and the
    LSTM forward/backward over as many of that minibatch's pieces (shortest
    first) as fit the time budget, scaled to the whole update by step count."""
    from oracle import (adam as oadam, gae as ogae, ingest as oing, is_weight as ois, lstm as olstm, pack as opack,
                        ppo_loss as oloss)
    from paper_2210_05064_amd import workloads as wl
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
    x_rows = opack.gather_rows(ro["obs"], meta["gather_idx"])
    t_pack = time.perf_counter() - t0
    M = meta["M"]
    W = olstm.weights_f64(ro["weights"])
    rng = np.random.default_rng(0)
    grads = olstm.zero_grads(W)
    steps = 0
    t0 = time.perf_counter()
    for j in range(meta["n_seq"] - 1, -1, -1):          # shortest pieces first
        f0, n = int(meta["seq_first"][j]), int(meta["seq_len"][j])
        u, v, saved = olstm.piece_forward(ro["obs"][f0:f0 + n], W)
        olstm.piece_backward(rng.standard_normal(u.shape) / M, rng.standard_normal(n) / M, W, saved, grads)
        steps += n
        if time.perf_counter() - t0 > budget_s:
            break
    t_lstm = (time.perf_counter() - t0) * M / steps
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
    t_update = t_ingest + t_gae + E * B * (t_pack + t_lstm + t_loss + t_adam)
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {
        "value": S / t_update, "unit": "env-steps/s", "cores": int(cores), "kind": "oracle",
        "sample": (f"bucketing of the arrival-order buffer ({t_ingest:.2f}s); GAE and importance weights on all {S} steps ({t_gae:.2f}s); packing ({t_pack:.2f}s) and loss ({t_loss:.2f}s) of one "
                   f"minibatch of {M} rows in full; LSTM fwd+bwd on {steps} steps of that minibatch's shortest "
                   f"pieces, scaled to {M} rows ({t_lstm:.1f}s); Adam step on all weights ({t_adam:.2f}s); "
                   f"update = bucketing + GAE + {E}x{B} minibatches"),
    }


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

    w = wl.WORKLOADS[args.workload]
    ro = wl.make_rollout(w, seed=args.seed)
    # the loss carries VER's truncated importance weight, and the optimiser runs inside the update: Adam with the paper's cosine schedule over its 500 M training steps
    learner = Learner(ro, adam_total_steps=max(1, int(500e6 // ro["S"])) * w.epochs * w.minibatches, max_is=MAX_IS,
                      arrival=None if args.env_major else wl.arrival_order(ro["env_off"], seed=args.seed + 1))
    learner.set_logp_old(collection_logp(ro, learner.compute, learner.x_bf16))
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        learner.update()
    torch.cuda.synchronize()
    if learner.lstm_timed_out() or learner.gae_timed_out():
        print("device-side wait timed out during warm-up", file=sys.stderr)
        sys.exit(4)

    rec_mask = (1 << ver.PROF_CLASSES.index("lstm_rec_fwd")) | (1 << ver.PROF_CLASSES.index("lstm_rec_bwd"))
    ver.ver_profile_enable(rec_mask)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        learner.update()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = ver.ver_profile_read()
    ver.ver_profile_enable(0)
    if learner.lstm_timed_out() or learner.gae_timed_out():
        print("device-side wait timed out during the timed region: results are invalid", file=sys.stderr)
        sys.exit(4)
    scalars = learner.scalars.cpu().numpy().tolist()
    t_max = int(learner.info[1].item())

    # every kernel class once more, for the breakdown (untimed)
    ver.ver_profile_enable((1 << len(ver.PROF_CLASSES)) - 1)
    learner.update()
    torch.cuda.synchronize()
    full = ver.ver_profile_read()
    ver.ver_profile_enable(0)

    S, M, H = learner.S, learner.M, w.hidden
    ms_per_step = 1e3 * elapsed / args.steps
    dom = max(("lstm_rec_fwd", "lstm_rec_bwd"), key=lambda k: prof[k][0])
    dom_ms, dom_n = prof[dom]
    # recurrent product of one layer over all timesteps of a minibatch: 2 * (4H x H) * rows.  With two layers one
    # launch runs both time loops and the projection between them (the same number of FLOPs again).
    flops_per_launch = 8.0 * H * H * M * (3 if w.n_layers == 2 else 1)
    achieved = flops_per_launch / (dom_ms / dom_n * 1e-3) / 1e12
    dtype = "bf16" if learner.compute else "f32"
    out = {
        "metric": "learner env-steps/sec per PPO update (1 MI355X)",
        "value": S / (elapsed / args.steps), "unit": "env-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": w.name, "n_envs": w.n_envs, "rollout_steps": S, "input_dim": w.input_dim,
                   "lstm": f"{w.n_layers}x{w.hidden}", "policy": "categorical" if w.dist == 0 else "gaussian",
                   "act_dim": w.act_dim, "epochs": w.epochs, "minibatches": w.minibatches,
                   "rows_per_minibatch": M, "seed": args.seed},
        "step_passes_per_sec": S * w.epochs / (elapsed / args.steps),
        "roofline": {"bound": "mfma", "kernel": dom,
                     "kernel_symbol": ("lstm_pipe_" if w.n_layers == 2 else "lstm_rec_") + dom[-3:] + "_kernel",
                     "achieved": achieved, "peak": PEAK_TFLOPS[dtype],
                     "unit": "TFLOP/s", "frac": achieved / PEAK_TFLOPS[dtype],
                     "traffic": MEASURED_TRAFFIC.get((w.name, dom)),
                     "avg_launch_ms": dom_ms / dom_n, "launches": dom_n, "flops_per_launch": flops_per_launch,
                     "last_minibatch_T_max": t_max},
        "kernel_ms_per_update": {k: round(v[0], 4) for k, v in full.items()},
        "kernel_launches_per_update": {k: v[1] for k, v in full.items()},
        "loss_scalars_last_minibatch": dict(zip(["total", "policy", "value", "entropy", "approx_kl", "clip_frac"],
                                                scalars)),
    }
    if not args.no_replica:
        # the HBM-bound kernels once more on gigabyte-sized replicas of the workload (untimed part of the run): at the
        # workload's own sizes they sit at the launch-latency floor, which says nothing about the kernels
        del learner
        torch.cuda.empty_cache()
        try:
            from paper_2210_05064_amd import hbm_replica
            out["hbm_replica"] = [{k: r[k] for k in ("kernel", "shape", "bytes", "ms", "achieved", "peak", "unit", "frac")}
                                  for r in hbm_replica.run(seed=args.seed + 3000, reps=4)]
        except Exception as e:   # the headline figures above do not depend on this part
            out["hbm_replica_error"] = repr(e)
    if args.cpu_budget > 0:
        out["cpu_baseline"] = cpu_baseline(ro, args.cpu_budget)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
