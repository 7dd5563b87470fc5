"""Pins for the GAE oracle: hand-worked values, brute force, closed forms,
invariants.  CPU only."""
import os

import numpy as np
import pytest

from oracle.gae import gae

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "gae_hand_example.txt")


def ragged(rng, n_envs=5, max_len=17, p_done=0.2, zero_len_env=True):
    L = rng.integers(1, max_len + 1, size=n_envs)
    if zero_len_env:
        L[1] = 0
    off = np.concatenate([[0], np.cumsum(L)]).astype(np.int32)
    S = int(off[-1])
    return dict(r=rng.standard_normal(S), v=rng.standard_normal(S),
                d=(rng.random(S) < p_done).astype(np.uint8), lv=rng.standard_normal(n_envs), off=off)


def test_hand_worked_example():
    params, rows = {}, []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if len(tok) == 2:
            params[tok[0]] = float(tok[1])
        else:
            rows.append([float(x) for x in tok])
    rows = np.array(rows)
    adv, ret = gae(rows[:, 0], rows[:, 1], rows[:, 2].astype(np.uint8), [params["last_value"]],
                   [0, len(rows)], params["gamma"], params["lambda"])
    np.testing.assert_allclose(adv, rows[:, 3], rtol=0, atol=1e-15)
    np.testing.assert_allclose(ret, rows[:, 4], rtol=0, atol=1e-15)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_brute_force_sum_of_td_errors(seed):
    """A_t = sum_{l=0}^{e-t} (gamma*lambda)^l delta_{t+l}, e = first done at or
    after t inside the stretch, else the stretch's last step."""
    rng = np.random.default_rng(seed)
    x = ragged(rng)
    gamma, lam = 0.97, 0.9
    adv, ret = gae(x["r"], x["v"], x["d"], x["lv"], x["off"], gamma, lam)
    for i in range(len(x["off"]) - 1):
        lo, hi = x["off"][i], x["off"][i + 1]
        for t in range(lo, hi):
            e = t
            while e < hi - 1 and not x["d"][e]:
                e += 1
            total = 0.0
            for k in range(t, e + 1):
                if x["d"][k]:
                    nxt = 0.0
                elif k == hi - 1:
                    nxt = x["lv"][i]
                else:
                    nxt = x["v"][k + 1]
                delta = x["r"][k] + gamma * nxt - x["v"][k]
                total += (gamma * lam) ** (k - t) * delta
            assert abs(adv[t] - total) < 1e-12
            assert abs(ret[t] - (total + x["v"][t])) < 1e-12


def test_lambda_zero_is_td_error():
    rng = np.random.default_rng(3)
    x = ragged(rng)
    adv, _ = gae(x["r"], x["v"], x["d"], x["lv"], x["off"], 0.9, 0.0)
    for i in range(len(x["off"]) - 1):
        lo, hi = x["off"][i], x["off"][i + 1]
        for k in range(lo, hi):
            nxt = 0.0 if x["d"][k] else (x["lv"][i] if k == hi - 1 else x["v"][k + 1])
            assert abs(adv[k] - (x["r"][k] + 0.9 * nxt - x["v"][k])) < 1e-13


def test_lambda_one_is_discounted_reward_to_go():
    rng = np.random.default_rng(4)
    x = ragged(rng)
    gamma = 0.93
    _, ret = gae(x["r"], x["v"], x["d"], x["lv"], x["off"], gamma, 1.0)
    for i in range(len(x["off"]) - 1):
        lo, hi = x["off"][i], x["off"][i + 1]
        for t in range(lo, hi):
            e = t
            while e < hi - 1 and not x["d"][e]:
                e += 1
            g = sum(gamma ** (k - t) * x["r"][k] for k in range(t, e + 1))
            if not x["d"][e]:
                g += gamma ** (e - t + 1) * x["lv"][i]
            assert abs(ret[t] - g) < 1e-12


def test_gamma_zero_and_all_done():
    rng = np.random.default_rng(5)
    x = ragged(rng)
    adv, _ = gae(x["r"], x["v"], x["d"], x["lv"], x["off"], 0.0, 0.95)
    np.testing.assert_allclose(adv, x["r"] - x["v"], atol=1e-15)
    adv, _ = gae(x["r"], x["v"], np.ones_like(x["d"]), x["lv"], x["off"], 0.99, 0.95)
    np.testing.assert_allclose(adv, x["r"] - x["v"], atol=1e-15)


def test_geometric_series():
    n, r, gamma, lam = 12, 0.7, 0.99, 0.95
    adv, _ = gae(np.full(n, r), np.zeros(n), np.zeros(n, np.uint8), [0.0], [0, n], gamma, lam)
    for t in range(n):
        m = n - t
        assert abs(adv[t] - r * (1 - (gamma * lam) ** m) / (1 - gamma * lam)) < 1e-12


def test_done_junction_equals_two_envs():
    """Two stretches glued into one environment with a done at the junction
    give the same advantages when the first stretch ends its episode."""
    rng = np.random.default_rng(6)
    x = ragged(rng, n_envs=2, zero_len_env=False)
    a = x["off"][1]
    x["d"][a - 1] = 1
    adv2, ret2 = gae(x["r"], x["v"], x["d"], x["lv"], x["off"], 0.99, 0.95)
    adv1, ret1 = gae(x["r"], x["v"], x["d"], x["lv"][1:], [0, x["off"][2]], 0.99, 0.95)
    np.testing.assert_allclose(adv1, adv2, atol=1e-15)
    np.testing.assert_allclose(ret1, ret2, atol=1e-15)


def test_env_permutation_permutes_outputs():
    rng = np.random.default_rng(7)
    x = ragged(rng)
    adv, _ = gae(x["r"], x["v"], x["d"], x["lv"], x["off"], 0.99, 0.95)
    n = len(x["off"]) - 1
    perm = rng.permutation(n)
    seg = lambda a: [a[x["off"][i]:x["off"][i + 1]] for i in perm]
    r2, v2, d2 = (np.concatenate(seg(x[k])) for k in ("r", "v", "d"))
    off2 = np.concatenate([[0], np.cumsum([x["off"][i + 1] - x["off"][i] for i in perm])])
    adv_p, _ = gae(r2, v2, d2, x["lv"][perm], off2, 0.99, 0.95)
    np.testing.assert_allclose(adv_p, np.concatenate(seg(adv)), atol=1e-15)


def test_equal_lengths_match_dense_textbook_recursion():
    """All L_i = T (fixed-length rollouts): a dense (T, N) backward recursion
    over whole columns must agree."""
    rng = np.random.default_rng(8)
    T, N, gamma, lam = 9, 4, 0.99, 0.95
    r, v = rng.standard_normal((T, N)), rng.standard_normal((T, N))
    d = (rng.random((T, N)) < 0.2)
    lv = rng.standard_normal(N)
    A = np.zeros((T + 1, N))
    vnext = np.vstack([v[1:], lv])
    for t in range(T - 1, -1, -1):
        A[t] = r[t] + gamma * vnext[t] * (~d[t]) - v[t] + gamma * lam * (~d[t]) * A[t + 1]
    flat = lambda a: a.T.reshape(-1)            # environment major
    adv, ret = gae(flat(r), flat(v), flat(d).astype(np.uint8), lv, np.arange(N + 1) * T, gamma, lam)
    np.testing.assert_allclose(adv, flat(A[:T]), atol=1e-14)
    np.testing.assert_allclose(ret, flat(A[:T] + v), atol=1e-14)


def test_planted_sign_error_would_be_caught():
    """The brute-force pin is sensitive: flipping the sign of the value
    baseline changes the result by far more than the test's tolerance."""
    rng = np.random.default_rng(9)
    x = ragged(rng)
    adv, _ = gae(x["r"], x["v"], x["d"], x["lv"], x["off"], 0.99, 0.95)
    wrong, _ = gae(x["r"], -x["v"], x["d"], x["lv"], x["off"], 0.99, 0.95)
    assert np.max(np.abs(adv - wrong)) > 1e-3
