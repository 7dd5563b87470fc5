"""Pins of the learned-entropy-coefficient oracle (oracle/entropy_coef.py): a hand-worked example, torch's
autograd with detach() as the stop-gradient operator, invariants against the fixed-coefficient loss, and a
planted mistake."""
import os

import numpy as np
import pytest
import torch

from oracle import entropy_coef as oec, ppo_loss as oloss

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "entropy_coef_hand_example.txt")


def golden_rows():
    rows = [[float(x) for x in line.split()] for line in open(GOLDEN) if line.strip() and not line.startswith("#")]
    return [r for r in rows if len(r) == 6], [r for r in rows if len(r) == 2]


def test_hand_example():
    terms, proj = golden_rows()
    assert len(terms) == 2 and len(proj) == 4
    for alpha, H, lam, value, d_alpha, d_H in terms:
        got = oec.entropy_terms(alpha, H, lam)
        assert got == pytest.approx((value, d_alpha, d_H), rel=1e-12, abs=1e-15)
        assert oec.entropy_terms(alpha, H, lam, sign=-1.0)[1] == pytest.approx(-d_alpha)
    for alpha, want in proj:
        assert oec.project(alpha) == want


def case(dist, seed, M=37, A=5):
    rng = np.random.default_rng(seed)
    u, v = rng.standard_normal((M, A)), rng.standard_normal(M)
    log_std = 0.3 * rng.standard_normal(A)
    actions = rng.integers(0, A, M) if dist == 0 else rng.standard_normal((M, A))
    logp_old = rng.standard_normal(M) * 0.1 - (1.5 if dist == 0 else 6.0)
    adv, ret, w = rng.standard_normal(M), rng.standard_normal(M), rng.random(M)
    return u, v, log_std, actions, logp_old, adv, ret, w


@pytest.mark.parametrize("dist", [0, 1])
def test_against_torch_autograd_with_detach(dist):
    """The whole loss rebuilt from torch.distributions, with detach() where the paper puts the stop gradient:
    autograd's gradients for the head outputs, log_std and alpha."""
    u, v, log_std, actions, logp_old, adv, ret, w = case(dist, 3 + dist)
    alpha, lam, clip, vc = 0.07, 0.4, 0.2, 0.5
    tu = torch.tensor(u, requires_grad=True)
    tv = torch.tensor(v, requires_grad=True)
    tls = torch.tensor(log_std, requires_grad=True)
    ta = torch.tensor(alpha, dtype=torch.float64, requires_grad=True)
    tw = torch.tensor(w)
    if dist == 0:
        d = torch.distributions.Categorical(logits=tu)
        logp, ent = d.log_prob(torch.tensor(actions)), d.entropy()
    else:
        d = torch.distributions.Normal(tu, torch.exp(tls))
        logp, ent = d.log_prob(torch.tensor(actions)).sum(1), d.entropy().sum(1)
    rho = torch.exp(logp - torch.tensor(logp_old))
    tadv = torch.tensor(adv)
    pol = (tw * -torch.minimum(rho * tadv, torch.clamp(rho, 1 - clip, 1 + clip) * tadv)).mean()
    val = (tw * 0.5 * (tv - torch.tensor(ret)) ** 2).mean()
    H = (tw * ent).mean()
    total = pol + vc * val + ta * (lam - H.detach()) - ta.detach() * H
    total.backward()
    sc, d_u, d_v, d_ls, d_alpha = oec.ppo_loss_learned_entropy(dist, u, v, log_std, actions, logp_old, adv, ret, clip,
                                                                vc, alpha, lam, w)
    assert sc["total"] == pytest.approx(total.item(), rel=1e-12)
    assert d_alpha == pytest.approx(ta.grad.item(), rel=1e-12)
    np.testing.assert_allclose(d_u, tu.grad.numpy(), rtol=1e-9, atol=1e-14)
    np.testing.assert_allclose(d_v, tv.grad.numpy(), rtol=1e-9, atol=1e-14)
    if dist == 1:
        np.testing.assert_allclose(d_ls, tls.grad.numpy(), rtol=1e-9, atol=1e-14)


@pytest.mark.parametrize("dist", [0, 1])
def test_policy_sees_a_fixed_coefficient(dist):
    """With alpha held constant the policy's gradients are those of the fixed-coefficient loss at c_e = alpha,
    whatever the target; the total differs by alpha*(lambda - H) exactly; d_alpha ignores alpha."""
    u, v, log_std, actions, logp_old, adv, ret, w = case(dist, 11)
    for alpha, lam in [(1e-3, 0.0), (0.3, -2.0)]:
        ref_sc, ref_du, ref_dv, ref_dls = oloss.ppo_loss(dist, u, v, log_std, actions, logp_old, adv, ret, 0.2, 0.5, alpha, w)
        sc, d_u, d_v, d_ls, d_alpha = oec.ppo_loss_learned_entropy(dist, u, v, log_std, actions, logp_old, adv, ret, 0.2,
                                                                    0.5, alpha, lam, w)
        assert np.array_equal(d_u, ref_du) and np.array_equal(d_v, ref_dv) and np.array_equal(d_ls, ref_dls)
        H = ref_sc["entropy"]
        assert sc["total"] == pytest.approx(ref_sc["total"] + alpha * (lam - H), rel=1e-13)
        assert d_alpha == pytest.approx(lam - H, rel=1e-13)
        for k in ("policy", "value", "entropy", "approx_kl", "clip_frac"):
            assert sc[k] == ref_sc[k]


def test_entropy_at_target_gives_no_gradient_to_alpha():
    # 4 uniform logits: entropy log 4 in every row
    M = 6
    u = np.zeros((M, 4))
    sc, _, _, _, d_alpha = oec.ppo_loss_learned_entropy(0, u, np.zeros(M), None, np.zeros(M, np.int64), np.full(M, -np.log(4)),
                                                        np.ones(M), np.zeros(M), 0.2, 0.5, 0.01, target=np.log(4.0))
    assert abs(d_alpha) < 1e-15
    assert sc["total"] == pytest.approx(-1.0 - 0.01 * np.log(4.0))     # ratio 1, advantage 1, value loss 0


def test_finite_difference_in_alpha_holds_entropy_constant():
    """d_alpha is the slope of the value in alpha with H frozen: the expression is linear in alpha with slope
    (lambda - H) - H when nothing is frozen, so a naive finite difference must NOT match (planted mistake:
    forgetting the stop gradient on alpha in the second term)."""
    alpha, H, lam, e = 0.2, 1.3, 0.5, 1e-6
    value = lambda a: oec.entropy_terms(a, H, lam)[0]
    naive = (value(alpha + e) - value(alpha - e)) / (2 * e)
    d_alpha = oec.entropy_terms(alpha, H, lam)[1]
    assert naive == pytest.approx(lam - 2 * H, rel=1e-6)
    assert d_alpha == pytest.approx(lam - H) and abs(d_alpha - naive) > 1.0


def test_projection_properties():
    rng = np.random.default_rng(0)
    for a in rng.standard_normal(50):
        p = oec.project(a)
        assert 1e-4 <= p <= 1.0 and oec.project(p) == p
        if 1e-4 <= a <= 1.0:
            assert p == a
