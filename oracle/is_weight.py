"""CPU oracle: the truncated importance weight of VER's biased sampling.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file;
it shares no code with the HIP kernels.

What it follows: with variable experience rollouts an environment contributes
as many steps as it managed to simulate, so fast environments are
over-represented in the batch; the paper corrects for this with a truncated
importance-sampling weight with a maximum of 1.0 (section 4 "Training";
appendix hyper-parameter table: importance sampling yes, maximum 1.0).  The
formula is not given.  Reading taken: every step of environment i carries

    w_i = min(max_is, (S / N) / L_i)

the ratio of the share every environment would have had with equal-length
rollouts (S/N of the S collected steps, N environments, empty ones counted) to
the share it actually has (L_i steps); constant within an environment; it
multiplies the per-step loss terms (the loss's per-row weight).  Environments
with fewer steps than the average would get a weight above 1 and are truncated
to max_is.
"""
import numpy as np


def is_weights(env_off, max_is=1.0):
    """Per-step weight, flat [S] fp64, for the CSR stretch offsets env_off[N+1]."""
    env_off = np.asarray(env_off, np.int64)
    N, S = len(env_off) - 1, int(env_off[-1])
    w = np.zeros(S)
    for i in range(N):
        L = int(env_off[i + 1] - env_off[i])
        if L > 0:
            w[env_off[i]:env_off[i + 1]] = min(float(max_is), (S / N) / L)
    return w
