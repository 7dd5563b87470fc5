"""CPU oracle: advantages and returns over a ragged rollout buffer.

TEST INFRASTRUCTURE ONLY.  Plain fp64 loops, one environment at a time.  Nothing
in the product path may import this file; it shares no code with the HIP
kernels.

What it follows: the paper trains with PPO and Generalized Advantage
Estimation (section 4, "Training"), gamma = 0.99 and lambda = 0.95 (appendix,
hyper-parameter table).  The estimator itself is only cited there, so this is
the estimator of the cited GAE paper applied to what section 2.2 defines: each
environment contributes a stretch of L_i >= 0 consecutive steps, and episodes
may end at any step inside a stretch (the solid bars of figure 2B).

Readings taken where the paper is silent:
  * dones[k] = 1 means the episode ended WITH step k; nothing flows from step
    k+1 back into step k.
  * the value that follows the last collected step of environment i is passed
    in as last_values[i]; it is ignored when that last step ended an episode.
  * returns are adv + value (the value-function target); advantages are not
    normalised (hyper-parameter table: "Normalized Advantage: No").
"""
import numpy as np


def gae(rewards, values, dones, last_values, env_off, gamma, lam):
    """Returns (adv[S], ret[S]) in fp64.

    rewards, values: [S] floats; dones: [S] 0/1; last_values: [N];
    env_off: [N+1] exclusive prefix sum of the per-environment step counts.
    """
    r = np.asarray(rewards, np.float64)
    v = np.asarray(values, np.float64)
    d = np.asarray(dones)
    lv = np.asarray(last_values, np.float64)
    S = r.shape[0]
    adv = np.zeros(S, np.float64)
    ret = np.zeros(S, np.float64)
    n_envs = len(env_off) - 1
    for i in range(n_envs):
        next_value = lv[i]
        next_adv = 0.0
        for k in range(int(env_off[i + 1]) - 1, int(env_off[i]) - 1, -1):
            not_done = 0.0 if d[k] else 1.0
            delta = r[k] + gamma * not_done * next_value - v[k]
            a = delta + gamma * lam * not_done * next_adv
            adv[k] = a
            ret[k] = a + v[k]
            next_value = v[k]
            next_adv = a
    return adv, ret
