"""Pins of the optimiser oracle (oracle/adam.py): a hand-worked example, a library cross-check, closed forms,
invariants and a planted mistake.  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import adam as oadam

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "adam_hand_example.txt")


def test_hand_example():
    cfg, rows = {}, []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        parts = line.split()
        if len(parts) == 2:
            cfg[parts[0]] = float(parts[1])
        else:
            rows.append([float(x) for x in parts])
    p, m, v = [np.array([cfg["p0"]])], [np.zeros(1)], [np.zeros(1)]
    for step, g, m_ref, v_ref, p_ref in rows:
        p, m, v, _ = oadam.adam_step(p, [np.array([g])], m, v, int(step), cfg["lr"], cfg["beta1"], cfg["beta2"], cfg["eps"])
        assert m[0][0] == pytest.approx(m_ref, abs=1e-15)
        assert v[0][0] == pytest.approx(v_ref, abs=1e-15)
        assert p[0][0] == pytest.approx(p_ref, abs=1e-15)


def test_against_torch_adam_and_cosine_schedule():
    """torch.optim.Adam + CosineAnnealingLR on fp64 tensors, 7 steps, several tensor shapes."""
    rng = np.random.default_rng(0)
    shapes = [(5, 3), (7,), (1,), (4, 4, 2)]
    p0 = [rng.standard_normal(s) for s in shapes]
    tp = [torch.tensor(x.copy(), dtype=torch.float64, requires_grad=True) for x in p0]
    opt = torch.optim.Adam(tp, lr=2.5e-4, betas=(0.9, 0.999), eps=1e-8)
    total = 10
    sched = torch.optim.lr_scheduler.CosineAnnealingLR(opt, T_max=total, eta_min=0.0)
    p, m, v = [x.copy() for x in p0], [np.zeros(s) for s in shapes], [np.zeros(s) for s in shapes]
    for k in range(7):
        grads = [rng.standard_normal(s) * 10.0 ** rng.integers(-3, 2) for s in shapes]
        for t, g in zip(tp, grads):
            t.grad = torch.tensor(g)
        assert opt.param_groups[0]["lr"] == pytest.approx(oadam.cosine_lr(k, total, 2.5e-4), rel=1e-12)
        opt.step()
        sched.step()
        p, m, v, _ = oadam.adam_step(p, grads, m, v, k + 1, oadam.cosine_lr(k, total, 2.5e-4))
        for a, b in zip(p, tp):
            np.testing.assert_allclose(a, b.detach().numpy(), rtol=1e-12, atol=1e-15)


def test_against_torch_clipping():
    rng = np.random.default_rng(1)
    shapes = [(6, 2), (9,)]
    grads = [rng.standard_normal(s) * 3 for s in shapes]
    tg = [torch.tensor(g.copy(), dtype=torch.float64, requires_grad=True) for g in grads]
    for t, g in zip(tg, grads):
        t.grad = torch.tensor(g.copy())
    norm = float(torch.nn.utils.clip_grad_norm_(tg, 0.5))
    p = [np.zeros(s) for s in shapes]
    p1, m1, v1, n1 = oadam.adam_step(p, grads, [np.zeros(s) for s in shapes], [np.zeros(s) for s in shapes], 1, 1e-3,
                                     max_grad_norm=0.5)
    assert n1 == pytest.approx(norm, rel=1e-12)
    for mi, t in zip(m1, tg):   # m after one step = (1 - beta1) * clipped gradient
        np.testing.assert_allclose(mi / 0.1, t.grad.numpy(), rtol=1e-12)
    # below the threshold nothing changes
    p2, m2, _, _ = oadam.adam_step(p, grads, [np.zeros(s) for s in shapes], [np.zeros(s) for s in shapes], 1, 1e-3,
                                   max_grad_norm=1e6)
    for mi, g in zip(m2, grads):
        np.testing.assert_allclose(mi / 0.1, g, rtol=1e-15)


def test_closed_forms():
    # first step: p moves by lr * g / (|g| + eps) whatever the size of g
    for g in (1e-3, 0.5, 40.0, -7.0):
        p, _, _, _ = oadam.adam_step([np.array([1.0])], [np.array([g])], [np.zeros(1)], [np.zeros(1)], 1, 0.01, eps=1e-8)
        assert p[0][0] == pytest.approx(1.0 - 0.01 * g / (abs(g) + 1e-8), abs=1e-15)
    # constant gradient: every step moves by lr * sign(g) (eps -> 0), bias correction makes m-hat = g, v-hat = g^2
    p, m, v = [np.array([0.0])], [np.zeros(1)], [np.zeros(1)]
    for t in range(1, 6):
        p, m, v, _ = oadam.adam_step(p, [np.array([3.0])], m, v, t, 0.1, eps=0.0)
        assert p[0][0] == pytest.approx(-0.1 * t, abs=1e-14)
    # zero gradient from a zero state: nothing moves
    p, m, v, n = oadam.adam_step([np.array([2.0, -1.0])], [np.zeros(2)], [np.zeros(2)], [np.zeros(2)], 1, 0.1)
    assert n == 0.0 and np.all(p[0] == [2.0, -1.0]) and np.all(m[0] == 0) and np.all(v[0] == 0)
    # cosine schedule: endpoints, midpoint, clamping
    assert oadam.cosine_lr(0, 100, 2.5e-4) == pytest.approx(2.5e-4)
    assert oadam.cosine_lr(50, 100, 2.5e-4) == pytest.approx(1.25e-4)
    assert oadam.cosine_lr(100, 100, 2.5e-4) == pytest.approx(0.0, abs=1e-20)
    assert oadam.cosine_lr(250, 100, 2.5e-4, 1e-5) == pytest.approx(1e-5)
    assert oadam.cosine_lr(25, 100, 1.0) == pytest.approx(0.5 * (1 + math.cos(math.pi / 4)))


def test_invariants():
    rng = np.random.default_rng(2)
    g = [rng.standard_normal((8, 3)), rng.standard_normal(5)]
    z = lambda: [np.zeros((8, 3)), np.zeros(5)]
    p0 = [rng.standard_normal((8, 3)), rng.standard_normal(5)]
    # with eps = 0 the update does not depend on the scale of the gradients
    a, _, _, _ = oadam.adam_step(p0, g, z(), z(), 1, 0.01, eps=0.0)
    b, _, _, _ = oadam.adam_step(p0, [1000.0 * x for x in g], z(), z(), 1, 0.01, eps=0.0)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=1e-12)
    # tensors are independent without clipping: updating them one by one gives the same result
    c0, _, _, _ = oadam.adam_step(p0[:1], g[:1], z()[:1], z()[:1], 1, 0.01)
    c1, _, _, _ = oadam.adam_step(p0[1:], g[1:], z()[1:], z()[1:], 1, 0.01)
    full, _, _, _ = oadam.adam_step(p0, g, z(), z(), 1, 0.01)
    assert np.array_equal(full[0], c0[0]) and np.array_equal(full[1], c1[0])
    # clipped gradients have exactly the requested norm (up to the 1e-6 guard)
    _, m, _, n = oadam.adam_step(p0, g, z(), z(), 1, 0.01, max_grad_norm=0.25)
    assert oadam.global_norm([x / 0.1 for x in m]) == pytest.approx(0.25 * n / (n + 1e-6), rel=1e-12)


def test_planted_mistake_is_caught():
    """A step without bias correction (a plausible slip) must fail the torch cross-check."""
    g, p = np.array([0.3]), np.array([1.0])
    m = 0.1 * g
    v = 0.001 * g * g
    wrong = p - 1e-3 * m / (np.sqrt(v) + 1e-8)
    right, _, _, _ = oadam.adam_step([p], [g], [np.zeros(1)], [np.zeros(1)], 1, 1e-3)
    assert abs(wrong[0] - right[0][0]) > 1e-4


def test_projection_is_elementwise_clip():
    rng = np.random.default_rng(5)
    params = [rng.standard_normal((3, 4)), rng.standard_normal(1), rng.standard_normal(6)]
    out = oadam.project(params, [-np.inf, 1e-4, -0.5], [np.inf, 1.0, 0.5])
    assert np.array_equal(out[0], params[0])
    assert out[1][0] == min(max(params[1][0], 1e-4), 1.0)
    assert np.array_equal(out[2], np.clip(params[2], -0.5, 0.5))
    assert np.all(out[2] <= 0.5) and np.all(out[2] >= -0.5) and np.any(out[2] != params[2])
