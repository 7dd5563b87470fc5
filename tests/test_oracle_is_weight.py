"""Pins of the importance-weight oracle (oracle/is_weight.py): closed forms and the property that defines
the weight.  CPU only."""
import numpy as np

from oracle import is_weight as ois


def off(lengths):
    return np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)


def test_equal_lengths_need_no_correction():
    assert np.all(ois.is_weights(off([7, 7, 7, 7])) == 1.0)


def test_hand_example():
    # 4 environments, 24 steps: the average share is 6 steps.  Lengths 12, 6, 4, 2 -> 6/12, 6/6, 6/4 -> 1, 6/2 -> 1.
    w = ois.is_weights(off([12, 6, 4, 2]))
    assert np.allclose(w[:12], 0.5) and np.allclose(w[12:18], 1.0) and np.allclose(w[18:], 1.0)
    # a higher ceiling lets the slow environments through: 1.5 and min(3, 2.5)
    w = ois.is_weights(off([12, 6, 4, 2]), max_is=2.5)
    assert np.allclose(w[18:22], 1.5) and np.allclose(w[22:], 2.5)


def test_untruncated_weights_give_every_environment_the_same_total():
    """The defining property: without truncation the weighted number of steps of every non-empty environment is
    S/N, as if all had collected equally many."""
    rng = np.random.default_rng(0)
    lengths = rng.integers(0, 40, size=13)
    lengths[3] = 0                                   # an environment that contributed nothing
    o = off(lengths)
    w = ois.is_weights(o, max_is=np.inf)
    share = o[-1] / len(lengths)
    for i, L in enumerate(lengths):
        tot = w[o[i]:o[i + 1]].sum()
        assert (L == 0 and tot == 0) or abs(tot - share) < 1e-9


def test_truncation_only_lowers_and_never_exceeds_the_ceiling():
    rng = np.random.default_rng(1)
    o = off(rng.integers(1, 60, size=20))
    free, cut = ois.is_weights(o, np.inf), ois.is_weights(o, 1.0)
    assert np.all(cut <= 1.0) and np.all(cut <= free) and np.all(cut[free <= 1.0] == free[free <= 1.0])
    assert cut.sum() <= o[-1]                        # the effective batch never grows


def test_constant_within_an_environment_and_permutation():
    lengths = np.array([5, 17, 1, 9])
    o = off(lengths)
    w = ois.is_weights(o)
    for i in range(4):
        assert len(set(w[o[i]:o[i + 1]])) == 1
    perm = [2, 0, 3, 1]
    wp = ois.is_weights(off(lengths[perm]))
    op = off(lengths[perm])
    for j, i in enumerate(perm):
        assert wp[op[j]] == w[o[i]]
