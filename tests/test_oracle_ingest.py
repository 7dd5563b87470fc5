"""Pins of the ingestion oracle (oracle/ingest.py): a hand-worked example, a brute-force second routine, the
round trip through the seeded arrival-order generator (which is the inverse operation), the time-major
special case, and the counter check."""
import os

import numpy as np
import pytest

from oracle import ingest as oing
from paper_2210_05064_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ingest_hand_example.txt")


def test_hand_example():
    rows = {l.split()[0]: [int(x) for x in l.split()[1:]] for l in open(GOLDEN) if l.strip() and not l.startswith("#")}
    env_off, order, bad = oing.ingest(rows["arr_env"], 3)
    assert env_off.tolist() == rows["env_off"] and order.tolist() == rows["order"] and bad == 0


def brute(arr_env, N):
    """Second routine: walk the environments, collect each one's slots in arrival order."""
    order, off = [], [0]
    for i in range(N):
        order += [a for a, e in enumerate(arr_env) if e == i]
        off.append(len(order))
    return off, order


@pytest.mark.parametrize("seed,N,S", [(0, 1, 9), (1, 5, 40), (2, 17, 300), (3, 300, 200), (4, 4, 0)])
def test_against_brute_force(seed, N, S):
    rng = np.random.default_rng(seed)
    arr_env = rng.integers(0, N, S)
    env_off, order, _ = oing.ingest(arr_env, N)
    off, ref = brute(arr_env.tolist(), N)
    assert env_off.tolist() == off and order.tolist() == ref
    assert sorted(order.tolist()) == list(range(S))                       # a permutation
    for i in range(N):                                                    # stretches: right environment, arrival order kept
        seg = order[env_off[i]:env_off[i + 1]]
        assert np.all(arr_env[seg] == i) and np.all(np.diff(seg) > 0)


@pytest.mark.parametrize("name", ["tiny", "nav", "manip", "large"])
def test_round_trip_through_the_arrival_generator(name):
    """The generator scatters an environment-major rollout into arrival order; ingestion must give back exactly
    the rollout's offsets and every field in its original place."""
    ro = wl.make_rollout(wl.scaled(wl.WORKLOADS[name], hidden=16, input_dim=8), seed=5, with_states=False)
    arr_env, arr_t, csr_of_arrival = wl.arrival_order(ro["env_off"], seed=9, t_start=np.arange(ro["N"]) * 7)
    assert len(set(arr_env[:ro["N"]].tolist())) > 1 or ro["N"] == 1       # interleaved, not environment-major
    env_off, order, bad = oing.ingest(arr_env, ro["N"], arr_t)
    assert np.array_equal(env_off, ro["env_off"]) and bad == 0
    assert np.array_equal(csr_of_arrival[order], np.arange(ro["S"]))      # order inverts the scatter
    for k in ("rewards", "dones", "obs"):
        assert np.array_equal(oing.to_env_major(ro[k][csr_of_arrival], order), ro[k])


def test_time_major_equal_lengths():
    T, N = 6, 5
    env_off, order = oing.dense_order(T, N)
    arr_env = np.tile(np.arange(N), T)                                    # slot t*N + i holds environment i
    g_off, g_order, _ = oing.ingest(arr_env, N, np.repeat(np.arange(T), N))
    assert np.array_equal(env_off, g_off) and np.array_equal(order, g_order)
    grid = np.arange(T * N).reshape(T, N)                                 # a [T, N] field
    assert np.array_equal(oing.to_env_major(grid.reshape(-1), order).reshape(N, T), grid.T)


def test_counter_check_counts_breaks_inside_stretches_only():
    arr_env = [0, 1, 0, 1, 0, 2]
    assert oing.ingest(arr_env, 3, [5, 0, 6, 1, 7, 9])[2] == 0            # every environment counts up from its own start
    assert oing.ingest(arr_env, 3, [5, 0, 7, 1, 8, 9])[2] == 1            # environment 0 skipped a step
    assert oing.ingest(arr_env, 3, [5, 0, 6, 1, 6, 9])[2] == 1            # a repeated counter
    assert oing.ingest(arr_env, 3, [7, 1, 6, 0, 5, 9])[2] == 3            # both environments run backwards
