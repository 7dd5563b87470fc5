"""Pins for the minibatch-creation / packed-layout oracle: all integer, exact.
CPU only."""
import numpy as np
import pytest

from oracle import pack


def ragged(rng, n_envs=6, max_len=40, p_done=0.12, B=3):
    L = rng.integers(0, max_len + 1, size=n_envs)
    L[-1] += (-int(L.sum())) % B
    off = np.concatenate([[0], np.cumsum(L)]).astype(np.int32)
    S = int(off[-1])
    dones = (rng.random(S) < p_done).astype(np.uint8)
    key = rng.integers(0, 2 ** 32, size=S, dtype=np.uint64).astype(np.uint32)
    eps = (rng.random(n_envs) < 0.5).astype(np.uint8)
    return off, dones, key, eps


def test_figure_style_example():
    """A 4-environment buffer like the paper's figure 2B, small enough to list
    by hand: stretches of 5, 2, 4, 3 steps; episode ends after step 1 of env 0
    and after step 2 of env 2 -> 6 sequences."""
    off = [0, 5, 7, 11, 14]
    dones = np.zeros(14, np.uint8)
    dones[1] = 1          # env 0, t=1
    dones[9] = 1          # env 2, t=2
    first, length, eps = pack.find_sequences(dones, off)
    assert first == [0, 2, 5, 7, 10, 11]
    assert length == [2, 3, 2, 3, 1, 3]
    assert eps == [0, 1, 0, 0, 1, 0]
    # keys chosen so the random order is sequences 3, 0, 5, 1, 4, 2
    key = np.zeros(14, np.uint32)
    for rank, s in enumerate([3, 0, 5, 1, 4, 2]):
        key[first[s]] = 10 * rank
    # stream: [7 8 9][0 1][11 12 | 13][2 3 4][10][5 6], cut after 7 steps
    m0 = pack.pack_minibatch(dones, off, key, 2, 0)
    assert m0["K"] == 6 and m0["n_seq"] == 3 and m0["T_max"] == 3
    assert m0["seq_first"].tolist() == [7, 0, 11]
    assert m0["seq_len"].tolist() == [3, 2, 2]
    assert m0["batch_sizes"].tolist() == [3, 3, 1]
    assert m0["t_off"].tolist() == [0, 3, 6, 7]
    assert m0["gather_idx"].tolist() == [7, 0, 11, 8, 1, 12, 9]
    m1 = pack.pack_minibatch(dones, off, key, 2, 1)
    # pieces in stream order: [13] (tail of a split sequence), [2 3 4], [10], [5 6]
    assert m1["seq_first"].tolist() == [2, 5, 13, 10]
    assert m1["seq_len"].tolist() == [3, 2, 1, 1]
    assert m1["seq_is_ep_start"].tolist() == [1, 0, 0, 1]
    assert m1["batch_sizes"].tolist() == [4, 2, 1]
    assert m1["gather_idx"].tolist() == [2, 5, 13, 10, 3, 6, 4]


@pytest.mark.parametrize("seed", range(6))
def test_structure_invariants(seed):
    rng = np.random.default_rng(seed)
    B = 3
    off, dones, key, eps = ragged(rng, B=B)
    S = int(off[-1])
    M = S // B
    seen = []
    stream = []
    first, length, _ = pack.find_sequences(dones, off, eps)
    for s in pack.random_order(first, key):
        stream += list(range(first[s], first[s] + length[s]))
    assert sorted(stream) == list(range(S))
    for b in range(B):
        m = pack.pack_minibatch(dones, off, key, B, b, eps)
        g = m["gather_idx"]
        # exactly the stream positions of this minibatch
        assert sorted(g.tolist()) == sorted(stream[b * M:(b + 1) * M])
        seen += g.tolist()
        bs = m["batch_sizes"]
        assert np.all(np.diff(bs) <= 0) and bs.sum() == M and (M == 0 or bs[0] == m["n_seq"])
        assert np.all(np.diff(m["seq_len"]) <= 0) and m["seq_len"].sum() == M
        assert m["t_off"][-1] == M
        # row j of timestep t continues row j of timestep t-1, with no episode end in between
        for t in range(1, m["T_max"]):
            for j in range(bs[t]):
                p, q = m["t_off"][t] + j, m["t_off"][t - 1] + j
                assert g[p] == g[q] + 1 and dones[g[q]] == 0
        # a piece never crosses an environment boundary
        for f, n in zip(m["seq_first"], m["seq_len"]):
            i = np.searchsorted(off, f, side="right") - 1
            assert f + n <= off[i + 1]
        # episode-start flags: step after a done, or a flagged stretch start
        for f, e in zip(m["seq_first"], m["seq_is_ep_start"]):
            i = np.searchsorted(off, f, side="right") - 1
            if f == off[i]:
                assert e == eps[i]
            elif dones[f - 1]:
                assert e == 1
            else:
                assert e == 0       # tail of a split sequence
    assert sorted(seen) == list(range(S))


@pytest.mark.parametrize("seed", range(4))
def test_brute_force_second_routine(seed):
    """Re-derive one minibatch a different way: label every flat step with its
    stream position through per-step arithmetic, cut by position, then build
    the packed order by repeated max-selection."""
    rng = np.random.default_rng(100 + seed)
    B = 2
    off, dones, key, eps = ragged(rng, B=B)
    S = int(off[-1])
    M = S // B
    # sequence id of every step, by scanning
    seq_id = np.zeros(S, np.int64)
    sid = -1
    env_of = np.zeros(S, np.int64)
    for i in range(len(off) - 1):
        env_of[off[i]:off[i + 1]] = i
    for k in range(S):
        if k == off[env_of[k]] or dones[k - 1]:
            sid += 1
        seq_id[k] = sid
    K = sid + 1
    heads = [int(np.argmax(seq_id == s)) for s in range(K)]
    rank = sorted(range(K), key=lambda s: (int(key[heads[s]]), s))
    start_of = {}
    pos = 0
    for s in rank:
        start_of[s] = pos
        pos += int(np.sum(seq_id == s))
    stream_pos = np.array([start_of[seq_id[k]] + (k - heads[seq_id[k]]) for k in range(S)])
    for b in range(B):
        steps = [k for k in range(S) if b * M <= stream_pos[k] < (b + 1) * M]
        # pieces = maximal runs of steps of one sequence
        steps.sort(key=lambda k: stream_pos[k])
        runs = []
        for k in steps:
            if runs and runs[-1][-1] + 1 == k and seq_id[runs[-1][-1]] == seq_id[k]:
                runs[-1].append(k)
            else:
                runs.append([k])
        # repeated max-selection (first maximum wins -> stable)
        ordered = []
        rest = list(runs)
        while rest:
            best = max(range(len(rest)), key=lambda a: (len(rest[a]), -a))
            ordered.append(rest.pop(best))
        expect = []
        t = 0
        while True:
            row = [r[t] for r in ordered if len(r) > t]
            if not row:
                break
            expect += row
            t += 1
        m = pack.pack_minibatch(dones, off, key, B, b, eps)
        assert m["gather_idx"].tolist() == expect
        assert m["seq_first"].tolist() == [r[0] for r in ordered]
        assert m["seq_len"].tolist() == [len(r) for r in ordered]


def test_equal_lengths_identity_order_is_dense_block():
    """Fixed-length rollouts without episode ends and keys in environment
    order: minibatch b is the dense time-major (T, N/B) block of its envs."""
    T, N, B = 7, 6, 3
    off = np.arange(N + 1) * T
    dones = np.zeros(T * N, np.uint8)
    key = np.zeros(T * N, np.uint32)
    key[off[:-1]] = np.arange(N)
    n = N // B
    for b in range(B):
        m = pack.pack_minibatch(dones, off, key, B, b)
        assert m["n_seq"] == n and m["T_max"] == T
        for t in range(T):
            for j in range(n):
                assert m["gather_idx"][t * n + j] == off[b * n + j] + t


def test_degenerate_cases():
    # every step ends an episode: every sequence has length 1
    off = [0, 3, 3, 8]
    dones = np.ones(8, np.uint8)
    key = np.arange(8, dtype=np.uint32)[::-1].copy()
    m = pack.pack_minibatch(dones, off, key, 2, 0)
    assert m["K"] == 8 and m["n_seq"] == 4 and m["T_max"] == 1
    assert m["gather_idx"].tolist() == [7, 6, 5, 4]
    # one environment owns the whole budget, no episode end: K = 1, split by the cut
    m = pack.pack_minibatch(np.zeros(8, np.uint8), [0, 0, 8], np.zeros(8, np.uint32), 2, 1)
    assert m["K"] == 1 and m["n_seq"] == 1 and m["seq_first"].tolist() == [4]
    assert m["seq_is_ep_start"].tolist() == [0] and m["gather_idx"].tolist() == [4, 5, 6, 7]
    # done on the last step of a stretch does not open an empty sequence
    d = np.zeros(4, np.uint8)
    d[3] = 1
    first, length, _ = pack.find_sequences(d, [0, 4])
    assert first == [0] and length == [4]
    with pytest.raises(ValueError):
        pack.pack_minibatch(np.zeros(7, np.uint8), [0, 7], np.zeros(7, np.uint32), 2, 0)


def test_equal_keys_fall_back_to_discovery_order():
    off = [0, 2, 4, 6]
    dones = np.zeros(6, np.uint8)
    m = pack.pack_minibatch(dones, off, np.full(6, 5, np.uint32), 1, 0)
    assert m["seq_first"].tolist() == [0, 2, 4]


def test_initial_states_and_gather():
    rng = np.random.default_rng(0)
    st = rng.standard_normal((2, 10, 3))
    out = pack.initial_states(st, [4, 0, 7], [0, 1, 0])
    assert np.array_equal(out[:, 0], st[:, 4]) and np.all(out[:, 1] == 0) and np.array_equal(out[:, 2], st[:, 7])
    f = rng.standard_normal((10, 2))
    assert np.array_equal(pack.gather_rows(f, [3, 1]), f[[3, 1]])
