"""CPU oracle: VER minibatch creation and the packed-sequence layout.

TEST INFRASTRUCTURE ONLY.  Plain Python/numpy, integer work.  Nothing in the
product path may import this file; it shares no code with the HIP kernels.

What it follows (paper section 2.2, "Learning mini-batch creation" and
"Batching computation for learning", figure 2B/2C):
  * a new sequence starts at the start of an environment's stretch and at the
    step after an episode end, so N environments give K >= N sequences;
  * the K sequences are put in random order, the first S/B steps of that order
    are minibatch 0, the next S/B steps minibatch 1, and so on (equal sizes);
  * a minibatch is laid out so that all sequence elements of one timestep are
    contiguous and timesteps follow each other.

Readings taken where the paper is silent:
  * the random order is an input: one 32-bit key per step, only the key at a
    sequence's first step counts; order = ascending (key, discovery index);
  * a sequence that straddles a cut is split: its head closes one minibatch,
    its tail opens the next and is not an episode start;
  * inside a minibatch pieces are ordered by length, longest first, ties in
    random-order position (stable); that makes row j of timestep t the
    successor of row j of timestep t-1;
  * a stretch's first step is an episode start only if the caller says so
    (env_started_episode), because the previous rollout is not visible here;
  * B must divide S.
"""
import numpy as np


def find_sequences(dones, env_off, env_started_episode=None):
    """Sequences in discovery order (environment index, then time).

    Returns three int lists: first flat step, length, is-episode-start.
    """
    first, length, ep_start = [], [], []
    n_envs = len(env_off) - 1
    for i in range(n_envs):
        lo, hi = int(env_off[i]), int(env_off[i + 1])
        k = lo
        while k < hi:
            begin = k
            if begin == lo:
                starts_episode = 0 if env_started_episode is None else int(env_started_episode[i] != 0)
            else:
                starts_episode = 1                    # the step after an episode end
            while k < hi - 1 and not dones[k]:
                k += 1
            k += 1                                    # k-1 was the sequence's last step
            first.append(begin)
            length.append(k - begin)
            ep_start.append(starts_episode)
    return first, length, ep_start


def random_order(first, seq_key):
    """Sequence ids sorted by (key at the sequence's first step, id)."""
    ids = list(range(len(first)))
    ids.sort(key=lambda s: (int(seq_key[first[s]]), s))
    return ids


def pack_minibatch(dones, env_off, seq_key, n_minibatches, b, env_started_episode=None):
    """Metadata of minibatch b of n_minibatches.

    Returns a dict of int arrays:
      K            number of sequences in the whole buffer
      n_seq        pieces in this minibatch, T_max its longest piece
      seq_first    [n_seq] flat step of each piece's first step (sorted order)
      seq_len      [n_seq] piece lengths, non-increasing
      seq_is_ep_start [n_seq] 1 if the piece begins an episode
      batch_sizes  [T_max]   rows present at timestep t
      t_off        [T_max+1] exclusive prefix sum of batch_sizes
      gather_idx   [M]       packed row -> flat step
    """
    S = int(env_off[-1])
    if S % n_minibatches != 0:
        raise ValueError("the number of minibatches must divide the number of steps")
    M = S // n_minibatches
    first, length, ep_start = find_sequences(dones, env_off, env_started_episode)
    order = random_order(first, seq_key)

    lo, hi = b * M, (b + 1) * M
    pieces = []                                       # (first step, length, episode start)
    pos = 0                                           # position in the virtual step stream
    for s in order:
        begin, end = pos, pos + length[s]
        pos = end
        cut_lo, cut_hi = max(begin, lo), min(end, hi)
        if cut_lo >= cut_hi:
            continue
        head_kept = cut_lo == begin
        pieces.append((first[s] + (cut_lo - begin), cut_hi - cut_lo, ep_start[s] if head_kept else 0))

    # longest first; Python's sort is stable, so ties keep random-order position
    pieces.sort(key=lambda p: -p[1])
    n_seq = len(pieces)
    seq_first = np.array([p[0] for p in pieces], np.int32)
    seq_len = np.array([p[1] for p in pieces], np.int32)
    seq_eps = np.array([p[2] for p in pieces], np.uint8)
    t_max = int(seq_len[0]) if n_seq else 0
    batch_sizes = np.array([int(np.sum(seq_len > t)) for t in range(t_max)], np.int32)
    t_off = np.zeros(t_max + 1, np.int32)
    t_off[1:] = np.cumsum(batch_sizes)
    gather_idx = np.zeros(M, np.int32)
    for t in range(t_max):
        for j in range(int(batch_sizes[t])):
            gather_idx[t_off[t] + j] = seq_first[j] + t
    return {
        "K": len(first), "n_seq": n_seq, "T_max": t_max, "M": M,
        "seq_first": seq_first, "seq_len": seq_len, "seq_is_ep_start": seq_eps,
        "batch_sizes": batch_sizes, "t_off": t_off, "gather_idx": gather_idx,
    }


def gather_rows(field, gather_idx):
    """packed[p] = field[gather_idx[p]] for a per-step field."""
    return np.asarray(field)[np.asarray(gather_idx, np.int64)]


def initial_states(rnn_state, seq_first, seq_is_ep_start):
    """Initial recurrent state of every piece.

    rnn_state[l, k, :] is the state layer l had before step k at collection
    time.  A piece that begins an episode starts from zeros; any other piece
    starts from the stored state of its first step.  Returns [nl, n_seq, H].
    """
    st = np.asarray(rnn_state)
    out = st[:, np.asarray(seq_first, np.int64), :].copy()
    out[:, np.asarray(seq_is_ep_start) != 0, :] = 0
    return out
