"""CPU oracle: from the linear collection buffer to the environment-major ragged buffer.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file;
it shares no code with the HIP kernels.

What it follows: during collection the inference workers write every step of
experience into a linear buffer in GPU memory as it arrives (section 2.2
"Batching computation for learning"; the workers and their dynamic batching:
section 2.1), so steps of different environments are interleaved and
environment i ends up with however many steps L_i it managed (the variable
experience rollout).  The learning phase works on each environment's steps in
time order (sequences, GAE), i.e. on the buffer bucketed by environment.

Definition written out: slot a of the linear buffer holds a step of environment
arr_env[a]; an environment's steps arrive in time order (it cannot have two
steps outstanding).  The environment-major buffer lists environment 0's steps
in arrival order, then environment 1's, ...: order[k] is the arrival slot of
flat step k, env_off the exclusive prefix sum of the per-environment counts.
That is a stable sort of the slots by environment.  Optional per-step counters
arr_t (each environment's own step number) are only checked: inside a stretch
they must go up by exactly one.  With equal-length rollouts written time-major
(slot t*N + i) the same definition gives order[i*T + t] = t*N + i.
"""
import numpy as np


def ingest(arr_env, N, arr_t=None):
    """Returns (env_off[N+1] int64, order[S] int64, violations): order[k] = arrival slot of flat step k;
    violations = number of flat steps k that continue a stretch but whose counter is not the previous one + 1
    (0 when arr_t is None)."""
    arr_env = np.asarray(arr_env, np.int64)
    S = len(arr_env)
    counts = np.zeros(N, np.int64)
    for e in arr_env:
        counts[e] += 1
    env_off = np.zeros(N + 1, np.int64)
    env_off[1:] = np.cumsum(counts)
    order = np.argsort(arr_env, kind="stable")
    violations = 0
    if arr_t is not None:
        arr_t = np.asarray(arr_t, np.int64)
        for i in range(N):
            for k in range(env_off[i] + 1, env_off[i + 1]):
                if arr_t[order[k]] != arr_t[order[k - 1]] + 1:
                    violations += 1
    return env_off, order, violations


def dense_order(T, N):
    """Equal-length rollouts stored time-major: slot t*N + i is step t of environment i."""
    env_off = np.arange(N + 1, dtype=np.int64) * T
    order = np.empty(N * T, np.int64)
    for i in range(N):
        for t in range(T):
            order[i * T + t] = t * N + i
    return env_off, order


def to_env_major(field, order):
    """Per-step field in arrival order -> the same field in environment-major order."""
    return np.asarray(field)[np.asarray(order, np.int64)]
