"""Pins for the PPO-loss oracle: invariants of the clipped objective, closed
forms, a library autograd cross-check, finite differences.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import ppo_loss as pl

CLIP, CV, CE = 0.2, 0.5, 1e-2


def batch(rng, dist, M=13, A=None):
    A = A or (4 if dist == pl.CATEGORICAL else 3)
    u = rng.standard_normal((M, A))
    v = rng.standard_normal(M)
    ls = 0.3 * rng.standard_normal(A) if dist == pl.GAUSSIAN else None
    act = rng.integers(0, A, M) if dist == pl.CATEGORICAL else rng.standard_normal((M, A))
    adv = rng.standard_normal(M)
    ret = rng.standard_normal(M)
    logp = np.array([pl.row_logp_entropy(dist, u[p], act[p], ls)[0] for p in range(M)])
    return dict(u=u, v=v, ls=ls, act=act, adv=adv, ret=ret, logp=logp)


def run(dist, x, logp_old, adv=None, weight=None):
    return pl.ppo_loss(dist, x["u"], x["v"], x["ls"], x["act"], logp_old, x["adv"] if adv is None else adv,
                       x["ret"], CLIP, CV, CE, weight)


@pytest.mark.parametrize("dist", [pl.CATEGORICAL, pl.GAUSSIAN])
def test_ratio_one_invariant(dist):
    x = batch(np.random.default_rng(0), dist)
    s, d_u, d_v, d_ls = pl.ppo_loss(dist, x["u"], x["v"], x["ls"], x["act"], x["logp"], x["adv"], x["ret"],
                                    CLIP, CV, 0.0)
    M = len(x["v"])
    assert abs(s["policy"] + np.mean(x["adv"])) < 1e-14
    assert s["clip_frac"] == 0 and abs(s["approx_kl"]) < 1e-15
    for p in range(M):       # d policy / d logp = -A / M, chained through dlogp/du
        dlogp_du = pl.row_logp_entropy(dist, x["u"][p], x["act"][p], x["ls"])[2]
        np.testing.assert_allclose(d_u[p], -x["adv"][p] / M * dlogp_du, atol=1e-15)


@pytest.mark.parametrize("dist", [pl.CATEGORICAL, pl.GAUSSIAN])
def test_zero_advantage_invariant(dist):
    rng = np.random.default_rng(1)
    x = batch(rng, dist)
    s, d_u, _, d_ls = pl.ppo_loss(dist, x["u"], x["v"], x["ls"], x["act"], x["logp"] + rng.standard_normal(13),
                                  np.zeros(13), x["ret"], CLIP, CV, 0.0)
    assert s["policy"] == 0 and np.all(d_u == 0) and np.all(d_ls == 0)


def test_clip_regions():
    """rho>1+eps with A>0 and rho<1-eps with A<0 are clipped (flat, no
    gradient); rho>1+eps with A<0 and rho<1-eps with A>0 are not."""
    x = batch(np.random.default_rng(2), pl.CATEGORICAL, M=4)
    shift = np.array([-0.5, 0.5, -0.5, 0.5])          # rho = e^{+0.5}, e^{-0.5}, ...
    adv = np.array([1.5, -2.0, -0.7, 0.9])
    s, d_u, _, _ = run(pl.CATEGORICAL, x, x["logp"] + shift, adv=adv)
    rho = np.exp(-shift)
    expect = [-(1 + CLIP) * adv[0], -(1 - CLIP) * adv[1], -rho[2] * adv[2], -rho[3] * adv[3]]
    assert abs(s["policy"] - np.mean(expect)) < 1e-14
    assert s["clip_frac"] == 1.0
    ent_only = pl.ppo_loss(pl.CATEGORICAL, x["u"], x["v"], None, x["act"], x["logp"] + shift, np.zeros(4),
                           x["ret"], CLIP, CV, CE)[1]
    np.testing.assert_allclose(d_u[:2], ent_only[:2], atol=1e-16)   # clipped rows: entropy term only
    assert np.max(np.abs(d_u[2] - ent_only[2])) > 1e-3 and np.max(np.abs(d_u[3] - ent_only[3])) > 1e-3


def test_closed_forms():
    A = 4
    logp, ent = pl.row_logp_entropy(pl.CATEGORICAL, np.full(A, 0.37), 2, None)[:2]
    assert abs(logp + math.log(A)) < 1e-15 and abs(ent - math.log(A)) < 1e-15
    A = 11
    mu = np.linspace(-1, 1, A)
    logp, ent = pl.row_logp_entropy(pl.GAUSSIAN, mu, mu, np.zeros(A))[:2]
    assert abs(logp + 0.5 * A * math.log(2 * math.pi)) < 1e-13
    assert abs(ent - 0.5 * A * (1 + math.log(2 * math.pi))) < 1e-13
    x = batch(np.random.default_rng(3), pl.GAUSSIAN)
    x["ret"] = x["v"].copy()
    s, _, d_v, _ = run(pl.GAUSSIAN, x, x["logp"])
    assert s["value"] == 0 and np.all(d_v == 0)


@pytest.mark.parametrize("dist", [pl.CATEGORICAL, pl.GAUSSIAN])
def test_against_library_autograd(dist):
    rng = np.random.default_rng(4)
    x = batch(rng, dist, M=17)
    logp_old = x["logp"] + 0.2 * rng.standard_normal(17)
    wt = rng.random(17)
    s, d_u, d_v, d_ls = run(dist, x, logp_old, weight=wt)
    u = torch.tensor(x["u"], requires_grad=True)
    v = torch.tensor(x["v"], requires_grad=True)
    if dist == pl.CATEGORICAL:
        pi = torch.distributions.Categorical(logits=u)
        logp, ent = pi.log_prob(torch.tensor(x["act"])), pi.entropy()
        ls = None
    else:
        ls = torch.tensor(x["ls"], requires_grad=True)
        pi = torch.distributions.Normal(u, ls.exp())
        logp, ent = pi.log_prob(torch.tensor(x["act"])).sum(-1), pi.entropy().sum(-1)
    w = torch.tensor(wt)
    ratio = (logp - torch.tensor(logp_old)).exp()
    a = torch.tensor(x["adv"])
    lpi = -(w * torch.min(ratio * a, ratio.clamp(1 - CLIP, 1 + CLIP) * a)).mean()
    lv = (w * 0.5 * (v - torch.tensor(x["ret"])) ** 2).mean()
    total = lpi + CV * lv - CE * (w * ent).mean()
    total.backward()
    assert abs(s["total"] - total.item()) < 1e-13
    assert abs(s["policy"] - lpi.item()) < 1e-13 and abs(s["value"] - lv.item()) < 1e-13
    np.testing.assert_allclose(d_u, u.grad.numpy(), atol=1e-14)
    np.testing.assert_allclose(d_v, v.grad.numpy(), atol=1e-14)
    if ls is not None:
        np.testing.assert_allclose(d_ls, ls.grad.numpy(), atol=1e-14)
    assert abs(s["approx_kl"] - (torch.tensor(logp_old) - logp).mean().item()) < 1e-14
    assert s["clip_frac"] == ((ratio - 1).abs() > CLIP).double().mean().item()


@pytest.mark.parametrize("dist", [pl.CATEGORICAL, pl.GAUSSIAN])
def test_finite_differences(dist):
    rng = np.random.default_rng(5)
    x = batch(rng, dist, M=6)
    logp_old = x["logp"] + 0.1 * rng.standard_normal(6)
    _, d_u, d_v, d_ls = run(dist, x, logp_old)
    eps = 1e-6
    targets = [(x["u"], d_u), (x["v"], d_v)] + ([(x["ls"], d_ls)] if dist == pl.GAUSSIAN else [])
    for arr, g in targets:
        flat, gflat = arr.reshape(-1), g.reshape(-1)
        for idx in range(flat.size):
            keep = flat[idx]
            flat[idx] = keep + eps
            up = run(dist, x, logp_old)[0]["total"]
            flat[idx] = keep - eps
            dn = run(dist, x, logp_old)[0]["total"]
            flat[idx] = keep
            assert abs((up - dn) / (2 * eps) - gflat[idx]) < 1e-8
