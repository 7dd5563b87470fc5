"""Seeded synthetic ragged rollouts shaped like the paper's workloads.

This module only draws random inputs.  It holds none of the learner's
arithmetic (no GAE, no packing, no LSTM, no loss) and imports neither the HIP
binding nor the CPU oracle, so both can be fed from the same arrays.

What the shapes stand for (paper section 2.2 and the hyper-parameter table of
the appendix): N environments contribute a total budget of S = T x N steps
with no constraint on the per-environment count L_i; episodes end at arbitrary
steps inside a stretch; the policy is a multi-layer LSTM fed a visual
embedding concatenated with a small state vector; actions are categorical
(navigation) or independent Gaussians (manipulation).

Everything is numpy on the host; `seed` fixes every draw.
"""
from __future__ import annotations

import dataclasses
import numpy as np


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    n_envs: int            # N
    budget: int            # S (0 = sum of uniformly drawn lengths, Tiny only)
    len_lo: int            # Tiny: L_i ~ U{len_lo..len_hi}
    len_hi: int
    speed_sigma: float     # sigma of LogNormal(0, sigma) env speeds
    input_dim: int         # D
    n_layers: int          # nl
    hidden: int            # H
    dist: int              # 0 categorical, 1 diagonal Gaussian
    act_dim: int           # A
    p_done: float
    epochs: int            # E
    minibatches: int       # B
    bf16: bool             # LSTM contractions in bf16 (fp32 accumulate)
    gamma: float = 0.99    # discount (hyper-parameter table)
    lam: float = 0.95      # GAE parameter (hyper-parameter table)
    clip: float = 0.2      # PPO clip (hyper-parameter table)
    value_coef: float = 0.5
    entropy_coef: float = 1e-4   # fixed coefficient of the benchmark runs


WORKLOADS = {
    "tiny": Workload("tiny", 4, 0, 8, 24, 0.0, 32, 1, 64, 0, 4, 0.05, 1, 1, False),
    "nav": Workload("nav", 16, 2048, 0, 0, 0.5, 516, 2, 512, 0, 4, 1.0 / 500, 2, 2, False),
    "manip": Workload("manip", 16, 2048, 0, 0, 1.0, 532, 2, 512, 1, 11, 1.0 / 200, 2, 2, False),
    "large": Workload("large", 64, 8192, 0, 0, 0.75, 516, 2, 512, 0, 4, 1.0 / 500, 2, 4, True),
    "max": Workload("max", 256, 32768, 0, 0, 1.0, 1044, 2, 1024, 1, 11, 1.0 / 200, 4, 4, True),
}


def apportion_steps(budget: int, speeds: np.ndarray) -> np.ndarray:
    """Split `budget` steps over environments in proportion to their speeds.

    Every environment gets one step, the rest is split by largest remainder
    (ties to the lower index), so the counts sum to `budget` exactly.
    """
    n = len(speeds)
    if budget < n:
        raise ValueError("budget smaller than the number of environments")
    share = (budget - n) * speeds / speeds.sum()
    base = np.floor(share).astype(np.int64)
    left = int(budget - n - base.sum())
    frac = share - base
    order = np.lexsort((np.arange(n), -frac))   # largest fraction first, low index wins ties
    base[order[:left]] += 1
    lengths = base + 1
    assert lengths.sum() == budget
    return lengths.astype(np.int32)


def env_lengths(w: Workload, rng: np.random.Generator) -> np.ndarray:
    if w.budget == 0:
        lengths = rng.integers(w.len_lo, w.len_hi + 1, size=w.n_envs).astype(np.int32)
        # keep the total divisible by the number of minibatches
        lengths[-1] += (-int(lengths.sum())) % w.minibatches
        return lengths
    speeds = rng.lognormal(0.0, w.speed_sigma, size=w.n_envs)
    return apportion_steps(w.budget, speeds)


def xavier_uniform(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    bound = np.sqrt(6.0 / (rows + cols))
    return rng.uniform(-bound, bound, size=(rows, cols)).astype(np.float32)


def make_weights(w: Workload, rng: np.random.Generator, bias_scale: float = 0.0) -> dict:
    """Xavier-uniform matrices; biases 0 (or small normals when bias_scale > 0, so
    that tests see bias gradients that are not hidden by zero values)."""
    H, A = w.hidden, w.act_dim
    layers = []
    for l in range(w.n_layers):
        d_in = w.input_dim if l == 0 else H
        layers.append({
            "W_ih": xavier_uniform(rng, 4 * H, d_in),
            "W_hh": xavier_uniform(rng, 4 * H, H),
            "b_ih": (bias_scale * rng.standard_normal(4 * H)).astype(np.float32),
            "b_hh": (bias_scale * rng.standard_normal(4 * H)).astype(np.float32),
        })
    return {
        "layers": layers,
        "W_a": xavier_uniform(rng, A, H),
        "b_a": (bias_scale * rng.standard_normal(A)).astype(np.float32),
        "w_v": xavier_uniform(rng, 1, H).reshape(H),
        "b_v": (bias_scale * rng.standard_normal(1)).astype(np.float32),
        "log_std": np.zeros(A, np.float32) if bias_scale == 0.0
        else (bias_scale * rng.standard_normal(A)).astype(np.float32),
    }


def make_rollout(w: Workload, seed: int, *, with_states: bool = True,
                 bias_scale: float = 0.0) -> dict:
    """One ragged rollout buffer plus policy weights, all seeded.

    Layout: step k = env_off[i] + t is step t of environment i (environment
    major, time ascending).  `dones[k] = 1` means the episode ended with step
    k.  `rnn_h/rnn_c[l, k]` is the recurrent state layer l had *before* step k
    at collection time.  `seq_key[e]` holds one random 32-bit sort key per step
    for epoch e (only the key at a sequence's first step is used).
    `logp_noise` is what a caller adds to the collection-time log-probability
    so that the probability ratio is not identically one.
    """
    rng = np.random.default_rng(seed)
    L = env_lengths(w, rng)
    S = int(L.sum())
    N = w.n_envs
    env_off = np.zeros(N + 1, np.int32)
    env_off[1:] = np.cumsum(L)
    out = {
        "workload": w, "seed": seed, "L": L, "env_off": env_off, "S": S, "N": N,
        "rewards": (0.1 * rng.standard_normal(S)).astype(np.float32),
        "values": rng.standard_normal(S).astype(np.float32),
        "last_values": rng.standard_normal(N).astype(np.float32),
        "dones": (rng.random(S) < w.p_done).astype(np.uint8),
        "env_started_episode": (rng.random(N) < 0.25).astype(np.uint8),
        "obs": rng.standard_normal((S, w.input_dim), dtype=np.float32),
        "logp_noise": (0.1 * rng.standard_normal(S)).astype(np.float32),
        "seq_key": rng.integers(0, 2 ** 32, size=(w.epochs, S), dtype=np.uint64).astype(np.uint32),
    }
    if w.dist == 0:
        out["actions"] = rng.integers(0, w.act_dim, size=S).astype(np.int32)
    else:
        out["actions"] = rng.standard_normal((S, w.act_dim), dtype=np.float32)
    if with_states:
        shape = (w.n_layers, S, w.hidden)
        out["rnn_h"] = (0.1 * rng.standard_normal(shape, dtype=np.float32))
        out["rnn_c"] = (0.1 * rng.standard_normal(shape, dtype=np.float32))
    out["weights"] = make_weights(w, rng, bias_scale)
    return out


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (tests shrink H or S)."""
    return dataclasses.replace(w, **kw)


def arrival_order(env_off: np.ndarray, seed: int, t_start: np.ndarray | None = None):
    """A linear buffer as inference workers would fill it: the S steps of a rollout interleaved across
    environments, every environment's own steps in time order.

    Every step gets a seeded completion time (environment i's steps at the running sum of its own exponential
    step durations, so that fast and slow stretches alternate as in the paper's collection phase); the buffer
    is written in order of completion time.  Returns (arr_env[S], arr_t[S], csr_of_arrival[S]): the environment
    and the environment's own step counter of the step in arrival slot a (counters start at t_start[i], zero
    when omitted), and the flat environment-major index that step has in the buffer env_off describes (what
    a test needs to build the arrival-order copy of any per-step field: field_arrival = field_csr[csr_of_arrival]).
    """
    env_off = np.asarray(env_off, np.int64)
    N, S = len(env_off) - 1, int(env_off[-1])
    rng = np.random.default_rng(seed)
    when = np.empty(S)
    env = np.empty(S, np.int32)
    t = np.empty(S, np.int32)
    for i in range(N):
        a, b = int(env_off[i]), int(env_off[i + 1])
        when[a:b] = np.cumsum(rng.exponential(1.0 / max(b - a, 1), size=b - a))
        env[a:b] = i
        t[a:b] = np.arange(b - a) + (0 if t_start is None else int(t_start[i]))
    csr_of_arrival = np.argsort(when, kind="stable").astype(np.int32)
    return env[csr_of_arrival], t[csr_of_arrival], csr_of_arrival
