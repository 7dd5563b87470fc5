"""Roofline-scale replicas of the HBM-bound kernels of the learner step.

At the paper's sizes the scan, the gathers, the loss, the optimiser step and the bucketing touch
between 0.1 MB and 0.5 GB per launch: they finish in microseconds, at the launch-latency floor, out
of the caches, and their share of the HBM roofline says little about the kernels.  This module runs
each of them once more on an input with the same structure as the `max` workload (LogNormal(0, 1)
environment speeds, 128 steps per environment on average, episode ends with probability 1/200,
D = 1044, 2 x 1024 recurrent state, 11 Gaussian action dimensions) but enough environments, rows or
parameters that a launch moves gigabytes, and reports algorithmic bytes / launch time against the
8 TB/s peak.  Launch times are the library's own HIP events on the launch stream.

Inputs are seeded and drawn on the GPU (torch generator) or on the host (numpy), nothing is read
from disk.  `bench.py --hbm-replica` prints the result as one JSON line.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as ver
from . import workloads as wl

HBM_PEAK_GBPS = 8000.0   # MI355X, HBM3E


def _timed(cls: str, call, reps: int, warmup: int = 3):
    """Average milliseconds per launch group of profile class `cls` over `reps` calls of call()."""
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    ver.ver_profile_enable(1 << ver.PROF_CLASSES.index(cls))
    for _ in range(reps):
        call()
    torch.cuda.synchronize()
    ms, n = ver.ver_profile_read()[cls]
    ver.ver_profile_enable(0)
    return ms / reps, n // reps


def _row(kernel, shape, nbytes, ms, launches, formula):
    gbps = nbytes / (ms * 1e-3) / 1e9
    return {"kernel": kernel, "shape": shape, "bytes": int(nbytes), "bytes_formula": formula, "ms": round(ms, 4),
            "launches": int(launches), "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(gbps / HBM_PEAK_GBPS, 4)}


def _lengths(n_envs: int, budget: int, rng: np.random.Generator) -> np.ndarray:
    env_off = np.zeros(n_envs + 1, np.int32)
    env_off[1:] = np.cumsum(wl.apportion_steps(budget, rng.lognormal(0.0, 1.0, size=n_envs)))
    return env_off


SECTIONS = ("gae", "pack", "loss", "adam", "ingest")
F32 = dict(dtype=torch.float32, device="cuda")
I32 = dict(dtype=torch.int32, device="cuda")


def run(seed: int = 7000, reps: int = 10, scale: int = 1, only=None) -> list:
    """scale divides every replica's size (tests use a large divisor); only: subset of SECTIONS to run."""
    want = set(SECTIONS if only is None else only)
    assert want <= set(SECTIONS), f"sections are {SECTIONS}"
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    rng = np.random.default_rng(seed)
    randn = lambda *shape: torch.randn(*shape, generator=g, **F32)
    out = []
    w = wl.WORKLOADS["max"]
    if "gae" in want:
        _gae(out, w, g, rng, randn, reps, scale)
    if "pack" in want:
        _pack(out, w, g, rng, randn, reps, scale, seed)
    if "loss" in want:
        _loss(out, w, g, randn, reps, scale)
    if "adam" in want:
        _adam(out, randn, reps, scale)
    if "ingest" in want:
        _ingest(out, rng, reps, scale, seed)
    return out


def _gae(out, w, g, rng, randn, reps, scale):
    """Advantages and importance weights: 2^27 steps of 2^20 environments."""
    f32 = F32
    N, S = (1 << 20) // scale, (1 << 27) // scale
    env_off = torch.from_numpy(_lengths(N, S, rng)).cuda()
    rewards, values, last_values = 0.1 * randn(S), randn(S), randn(N)
    dones = (torch.rand(S, generator=g, device="cuda") < w.p_done).to(torch.uint8)
    adv, ret = torch.empty(S, **f32), torch.empty(S, **f32)
    ws = ver.workspace(ver.ver_gae_workspace_bytes(S))
    ms, n = _timed("gae", lambda: ver.ver_gae(rewards, values, dones, last_values, env_off, N, S, w.gamma, w.lam,
                                              adv, ret, ws), reps)
    out.append(_row("gae_kernel", f"N={N} S={S}", 17 * S + 8 * N, ms, n, "17 B/step + 8 B/environment"))
    del rewards, values, dones, adv, ws
    ms, n = _timed("is_weight", lambda: ver.ver_is_weight(env_off, N, S, 1.0, ret), reps)
    out.append(_row("is_weight_mark_kernel + is_weight_fill_kernel", f"N={N} S={S}", 4 * S + 4 * N, ms, n, "4 B/step written + 4 B/environment"))
    del ret, env_off, last_values
    torch.cuda.empty_cache()



def _pack(out, w, g, rng, randn, reps, scale, seed):
    """Minibatch gather and the gathers of the bucketing: one minibatch of 2^18 rows."""
    f32, i32 = F32, I32
    N, S = 2048 // scale, (1 << 18) // scale
    D, A, H, nl = w.input_dim, w.act_dim, w.hidden, w.n_layers
    env_off_h = _lengths(N, S, rng)
    env_off = torch.from_numpy(env_off_h).cuda()
    dones = (torch.rand(S, generator=g, device="cuda") < w.p_done).to(torch.uint8)
    started = (torch.rand(N, generator=g, device="cuda") < 0.25).to(torch.uint8)
    seq_key = torch.randint(-2 ** 31, 2 ** 31 - 1, (S,), generator=g, **i32)
    obs, actions = randn(S, D), randn(S, A)
    logp, adv, ret, isw = randn(S), randn(S), randn(S), torch.rand(S, generator=g, **f32)
    rnn_h, rnn_c = 0.1 * randn(nl, S, H), 0.1 * randn(nl, S, H)
    cap = min(S, 16384)
    o = dict(info=torch.zeros(4, **i32), seq_first=torch.empty(S, **i32), seq_len=torch.empty(S, **i32),
             seq_is_ep_start=torch.empty(S, dtype=torch.uint8, device="cuda"), batch_sizes=torch.empty(S, **i32),
             t_off=torch.empty(S + 1, **i32), gather_idx=torch.empty(S, **i32),
             obs_packed=torch.empty((S, D), dtype=torch.bfloat16, device="cuda"), actions_packed=torch.empty((S, A), **f32),
             logp_old_packed=torch.empty(S, **f32), adv_packed=torch.empty(S, **f32), ret_packed=torch.empty(S, **f32),
             is_weight_packed=torch.empty(S, **f32), h0=torch.empty((nl, cap, H), **f32), c0=torch.empty((nl, cap, H), **f32))
    ws = ver.workspace(ver.ver_pack_workspace_bytes(N, S, 1))
    args = dict(dones=dones, env_off=env_off, env_started_episode=started, seq_key=seq_key, N=N, S=S, B=1, b=0,
                obs=obs, D=D, obs_packed_bf16=1, actions=actions, act_bytes=4 * A, logp_old=logp, adv=adv, ret=ret,
                is_weight=isw, rnn_h=rnn_h, rnn_c=rnn_c, n_layers=nl, H=H, seq_cap=cap, workspace=ws, **o)
    ver.ver_pack_minibatch(**args)
    n_seq = int(o["info"][0].item())
    args["index_ready"] = 1
    ms, n = _timed("pack_gather", lambda: ver.ver_pack_minibatch(**args), reps)
    per_row = 4 + 6 * D + 8 * A + 4 * 8
    out.append(_row("pack_gather_kernel", f"M={S} D={D} bf16 rows, {n_seq} pieces", per_row * S + min(n_seq, cap) * nl * H * 16,
                    ms, n, "per row: index 4 + observation 4D read, 2D written + action 2*4A + four scalars 2*4 each; "
                           "per piece: h and c of every layer read and written"))
    del rnn_h, rnn_c, o, args, logp, adv, ret, isw, actions
    order = torch.from_numpy(wl.arrival_order(env_off_h, seed=seed + 1)[2]).cuda()
    dst = torch.empty_like(obs)
    ms, n = _timed("ingest", lambda: ver.ver_ingest_gather(order, S, obs, dst), reps)
    out.append(_row("ingest_gather_kernel", f"S={S} rows of {4 * D} bytes", (8 * D + 4) * S, ms, n, "row read + row written + index 4"))
    del obs, dst, order
    torch.cuda.empty_cache()



def _loss(out, w, g, randn, reps, scale):
    """Loss: 2^24 rows."""
    f32 = F32
    A = w.act_dim
    M = (1 << 24) // scale
    head, value, acts = randn(M, A), randn(M), randn(M, A)
    logp, adv, ret, isw = randn(M) - 15.0, randn(M), randn(M), torch.rand(M, generator=g, **f32)
    log_std, d_log_std = torch.zeros(A, **f32), torch.empty(A, **f32)
    d_head, d_value, scalars = torch.empty((M, A), **f32), torch.empty(M, **f32), torch.zeros(6, **f32)
    cfg = ver.ppo_cfg(w.clip, w.value_coef, w.entropy_coef, 1, A)
    ws = ver.workspace(ver.ver_ppo_loss_workspace_bytes(M, A))
    ms, n = _timed("ppo_loss", lambda: ver.ver_ppo_loss(cfg, M, head, value, log_std, acts, logp, adv, ret, isw, scalars,
                                                        d_head, d_value, d_log_std, ws), reps)
    out.append(_row("ppo_loss_kernel", f"M={M} Gaussian A={A}", (12 * A + 6 * 4) * M, ms, n,
                    "per row: mean, action read and gradient written 3*4A + value, old log-prob, advantage, return, "
                    "weight read and value gradient written 6*4"))
    del head, value, acts, logp, adv, ret, isw, d_head, d_value
    torch.cuda.empty_cache()



def _adam(out, randn, reps, scale):
    """Optimiser step: 8 tensors of 2^24 parameters."""
    f32 = F32
    P, T = (1 << 24) // scale, 8
    params = [0.05 * randn(P) for _ in range(T)]
    grads = [1e-3 * randn(P) for _ in range(T)]
    m, v = [torch.zeros(P, **f32) for _ in range(T)], [torch.zeros(P, **f32) for _ in range(T)]
    acfg = ver.adam_cfg(total_steps=1000)
    ws = ver.workspace(ver.ver_adam_workspace_bytes())
    step = [0]

    def adam():
        ver.ver_adam_step(acfg, params, grads, m, v, step[0], None, ws)
        step[0] += 1
    ms, n = _timed("adam", adam, reps)
    out.append(_row("adam_update_kernel", f"{T} tensors x {P}", 28 * P * T, ms, n, "28 B/parameter"))
    gn = torch.zeros(1, **f32)

    def adam_norm():
        ver.ver_adam_step(acfg, params, grads, m, v, step[0], gn, ws)
        step[0] += 1
    ms, n = _timed("adam", adam_norm, reps)
    out.append(_row("adam_sumsq+norm+update", f"{T} tensors x {P}", 32 * P * T, ms, n, "32 B/parameter (gradients read twice)"))
    del params, grads, m, v
    torch.cuda.empty_cache()



def _ingest(out, rng, reps, scale, seed):
    """Bucketing of the arrival-order buffer: 2^24 slots of 2^16 environments."""
    i32 = I32
    N, S = (1 << 16) // scale, (1 << 24) // scale
    env_off_h = _lengths(N, S, rng)
    arr_env, arr_t, _ = wl.arrival_order(env_off_h, seed=seed + 2)
    arr_env, arr_t = torch.from_numpy(arr_env).cuda(), torch.from_numpy(arr_t).cuda()
    env_off, order, info = torch.zeros(N + 1, **i32), torch.empty(S, **i32), torch.zeros(4, **i32)
    ws = ver.workspace(ver.ver_ingest_workspace_bytes(N, S))
    ms, n = _timed("ingest", lambda: ver.ver_ingest(arr_env, arr_t, N, S, env_off, order, info, ws), reps)
    passes = -(-int(N).bit_length() // 10)
    out.append(_row("ingest (sort by environment)", f"N={N} S={S}, {passes} passes", (20 * passes + 8) * S, ms, n,
                    "per pass: ids read twice, slots read once (not in the first pass), both written: 20 B/slot "
                    "(16 in the first); last kernel: ids, slots and step counters read: 12 B/slot"))
