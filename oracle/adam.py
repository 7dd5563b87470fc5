"""CPU oracle: the optimiser step that follows the backward pass.

TEST INFRASTRUCTURE ONLY.  fp64 numpy, one tensor at a time.  Nothing in the
product path may import this file; it shares no code with the HIP kernels.

What it follows: the paper trains with the Adam optimiser, an initial learning
rate of 2.5e-4 decayed to zero with a cosine schedule (section 4 "Training";
appendix, hyper-parameter table).  Adam is only cited, so this is Algorithm 1
of the cited Adam paper, bias-corrected:

    m <- beta1*m + (1-beta1)*g            v <- beta2*v + (1-beta2)*g*g
    mhat = m / (1 - beta1^t)              vhat = v / (1 - beta2^t)
    p <- p - lr * mhat / (sqrt(vhat) + eps)              t = 1, 2, ...

Readings taken where the paper is silent: beta1 = 0.9, beta2 = 0.999,
eps = 1e-8 (the defaults of the cited paper); no weight decay; the cosine
schedule is lr_k = lr_final + (lr_0 - lr_final) * (1 + cos(pi*k/K)) / 2 for the
k-th optimiser step counted from 0 (the first step uses lr_0; k is clamped to
K); gradient clipping is not mentioned: it is optional, by global 2-norm over
all tensors, g <- g * min(1, max_norm / (norm + 1e-6)), off when
max_norm <= 0.  A tensor may carry bounds (the learned entropy coefficient
does: appendix hyper-parameter table, bounds [1e-4, 1]); the reading is a
projection onto them after the step.
"""
import math
import numpy as np


def cosine_lr(k, total_steps, lr0, lr_final=0.0):
    """Learning rate of the k-th optimiser step (k = 0 for the first one)."""
    k = min(max(int(k), 0), int(total_steps))
    return lr_final + (lr0 - lr_final) * 0.5 * (1.0 + math.cos(math.pi * k / total_steps))


def global_norm(grads):
    return math.sqrt(sum(float(np.sum(np.asarray(g, np.float64) ** 2)) for g in grads))


def adam_step(params, grads, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8, max_grad_norm=0.0):
    """One step on lists of arrays; t = 1 for the first step.  Returns (params, m, v, grad_norm) as new fp64
    arrays; grad_norm is the global 2-norm before clipping."""
    norm = global_norm(grads)
    scale = 1.0
    if max_grad_norm > 0.0:
        scale = min(1.0, max_grad_norm / (norm + 1e-6))
    c1, c2 = 1.0 - beta1 ** t, 1.0 - beta2 ** t
    new_p, new_m, new_v = [], [], []
    for p, g, mi, vi in zip(params, grads, m, v):
        g = np.asarray(g, np.float64) * scale
        mi = beta1 * np.asarray(mi, np.float64) + (1.0 - beta1) * g
        vi = beta2 * np.asarray(vi, np.float64) + (1.0 - beta2) * g * g
        new_p.append(np.asarray(p, np.float64) - lr * (mi / c1) / (np.sqrt(vi / c2) + eps))
        new_m.append(mi)
        new_v.append(vi)
    return new_p, new_m, new_v, norm


def project(params, lower, upper):
    """Projection of every tensor onto its box after a step: lower[i] <= p <= upper[i] elementwise
    (-inf / +inf = unbounded)."""
    return [np.minimum(np.maximum(np.asarray(p, np.float64), lo), hi) for p, lo, hi in zip(params, lower, upper)]
