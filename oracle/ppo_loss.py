"""CPU oracle: PPO clipped-surrogate + value + entropy loss, row by row.

TEST INFRASTRUCTURE ONLY.  fp64, one minibatch row at a time.  Nothing in the
product path may import this file; it shares no code with the HIP kernels.

What it follows: the paper learns with PPO (section 2.2, "Learning method")
with clip 0.2, value-loss coefficient 0.5, no clipped value loss, no advantage
normalisation (appendix, hyper-parameter table) and, for the throughput
benchmarks, a fixed entropy coefficient of 1e-4 (appendix, "Hyperparamaters").
Actions are categorical for navigation and independent Gaussians for
manipulation (section 4, "Architecture").  The objective is only cited, so
this is the clipped surrogate of the cited PPO paper:

    rho = exp(logp - logp_old)
    L_pi = -mean( min(rho * A, clip(rho, 1-eps, 1+eps) * A) )
    L_v  =  mean( 0.5 * (v - R)^2 )
    total = L_pi + c_v * L_v - c_e * mean(entropy)

Readings taken where the paper is silent: the value loss carries the factor
1/2; means run over the M rows of the minibatch; the gradient through min/clip
is the gradient of whichever branch is selected, the unclipped branch winning
ties; the Gaussian's standard deviation is exp(log_std) with one
state-independent log_std per action dimension; an optional per-row weight
multiplies all three per-row terms (1 when absent).
"""
import math
import numpy as np

CATEGORICAL, GAUSSIAN = 0, 1
LOG_2PI = math.log(2.0 * math.pi)


def row_logp_entropy(dist, u, action, log_std):
    """Log-probability of `action` and the entropy for one row, plus their
    gradients w.r.t. the head output u (and log_std for the Gaussian)."""
    A = u.shape[0]
    if dist == CATEGORICAL:
        m = np.max(u)
        lse = m + math.log(np.sum(np.exp(u - m)))
        logq = u - lse                                   # log softmax
        q = np.exp(logq)
        a = int(action)
        logp = logq[a]
        ent = -np.sum(q * logq)
        dlogp_du = -q.copy()
        dlogp_du[a] += 1.0
        dent_du = -q * (logq + ent)
        return logp, ent, dlogp_du, dent_du, np.zeros(A), np.zeros(A)
    sigma = np.exp(log_std)
    zed = (np.asarray(action, np.float64) - u) / sigma
    logp = np.sum(-0.5 * zed * zed - log_std - 0.5 * LOG_2PI)
    ent = np.sum(log_std + 0.5 * (1.0 + LOG_2PI))
    dlogp_du = zed / sigma
    dlogp_dls = zed * zed - 1.0
    return logp, ent, dlogp_du, np.zeros(A), dlogp_dls, np.ones(A)


def ppo_loss(dist, u, v, log_std, actions, logp_old, adv, ret, clip, value_coef, entropy_coef,
             weight=None):
    """u [M, A] head outputs, v [M] values, packed rows.

    Returns (scalars, d_u [M, A], d_v [M], d_log_std [A]) with scalars a dict:
    total, policy, value, entropy, approx_kl, clip_frac.  The gradients are of
    `total`.
    """
    u = np.asarray(u, np.float64)
    v = np.asarray(v, np.float64)
    M, A = u.shape
    log_std = np.zeros(A) if log_std is None else np.asarray(log_std, np.float64)
    logp_old = np.asarray(logp_old, np.float64)
    adv = np.asarray(adv, np.float64)
    ret = np.asarray(ret, np.float64)
    d_u = np.zeros((M, A))
    d_v = np.zeros(M)
    d_log_std = np.zeros(A)
    s_pi = s_v = s_ent = s_kl = s_clipped = 0.0
    for p in range(M):
        w = 1.0 if weight is None else float(weight[p])
        logp, ent, dlogp_du, dent_du, dlogp_dls, dent_dls = row_logp_entropy(dist, u[p], actions[p], log_std)
        rho = math.exp(logp - logp_old[p])
        unclipped = rho * adv[p]
        clipped = min(max(rho, 1.0 - clip), 1.0 + clip) * adv[p]
        s_pi += -w * min(unclipped, clipped)
        s_v += w * 0.5 * (v[p] - ret[p]) ** 2
        s_ent += w * ent
        s_kl += logp_old[p] - logp
        s_clipped += 1.0 if abs(rho - 1.0) > clip else 0.0
        # d(-min(..))/dlogp: the unclipped branch carries gradient rho*A, the clipped one none
        dpi_dlogp = -adv[p] * rho if unclipped <= clipped else 0.0
        coef_logp = w * dpi_dlogp / M
        coef_ent = -entropy_coef * w / M
        d_u[p] = coef_logp * dlogp_du + coef_ent * dent_du
        d_log_std += coef_logp * dlogp_dls + coef_ent * dent_dls
        d_v[p] = value_coef * w * (v[p] - ret[p]) / M
    scalars = {
        "policy": s_pi / M, "value": s_v / M, "entropy": s_ent / M,
        "approx_kl": s_kl / M, "clip_frac": s_clipped / M,
    }
    scalars["total"] = scalars["policy"] + value_coef * scalars["value"] - entropy_coef * scalars["entropy"]
    return scalars, d_u, d_v, d_log_std
