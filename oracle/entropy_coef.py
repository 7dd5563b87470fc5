"""CPU oracle: the learned entropy coefficient of the training runs.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file;
it shares no code with the HIP kernels.

What it follows: instead of a fixed entropy coefficient the paper trains with a
minimum-entropy constraint whose coefficient alpha is learned (section 4
"Training"): with H the policy's entropy, lambda the target entropy and sg[.]
the stop-gradient operator it minimises

    alpha * (lambda - sg[H])  -  sg[alpha] * H

with lambda = 0, alpha initialised to 1e-3 and kept inside [1e-4, 1]
(appendix, hyper-parameter table).  So the policy sees an entropy bonus with
the current alpha as a constant, and alpha sees lambda - H as its gradient.

Readings taken where the paper is silent or at odds with itself:
  * H is the entropy term of the PPO loss: the (weighted) mean over the M rows
    of the minibatch, the same number the fixed-coefficient loss uses.
  * The expression replaces "- c_e * mean(entropy)" in the PPO total.
  * alpha itself is the parameter (no log / softplus parameterisation), one
    more tensor of the optimiser step, projected onto its bounds after the
    step: alpha <- min(max(alpha, lower), upper).
  * Sign of alpha's gradient.  Minimising the printed expression over alpha
    gives d/d alpha = lambda - H: alpha shrinks while the entropy is BELOW the
    target, which is the opposite of what a minimum-entropy constraint needs
    (the multiplier of a constraint H >= lambda ascends on alpha*(lambda - H)).
    The printed form is the default (sign = +1); sign = -1 hands the
    optimiser H - lambda instead, i.e. dual ascent.  The value of the
    expression and the policy's gradient do not depend on the sign.
"""
import numpy as np

from . import ppo_loss


def entropy_terms(alpha, H, target=0.0, sign=1.0):
    """Value of alpha*(target - sg[H]) - sg[alpha]*H and the two gradients it
    defines: d/d alpha (times `sign`) and d/dH (what the policy is given)."""
    value = alpha * (target - H) - alpha * H
    return value, sign * (target - H), -alpha


def project(alpha, lower=1e-4, upper=1.0):
    """Projection of the coefficient onto its bounds."""
    return min(max(float(alpha), float(lower)), float(upper))


def ppo_loss_learned_entropy(dist, u, v, log_std, actions, logp_old, adv, ret, clip, value_coef, alpha,
                             target=0.0, weight=None, sign=1.0):
    """The PPO loss with the learned coefficient: the fixed-coefficient loss at
    c_e = alpha (the policy treats alpha as a constant) plus alpha's own term.
    Returns (scalars, d_u, d_v, d_log_std, d_alpha)."""
    scalars, d_u, d_v, d_log_std = ppo_loss.ppo_loss(dist, u, v, log_std, actions, logp_old, adv, ret, clip,
                                                     value_coef, alpha, weight)
    H = scalars["entropy"]
    value, d_alpha, _ = entropy_terms(alpha, H, target, sign)
    scalars = dict(scalars)
    # the fixed-coefficient total already holds - alpha * H
    scalars["total"] = scalars["total"] + alpha * H + value
    return scalars, d_u, d_v, d_log_std, d_alpha
