"""ver_adam_step against the CPU oracle (oracle/adam.py, fp64).  The learning rate is large here so that the
update is far above the fp32 resolution of the parameters: what is compared is the arithmetic of the step
(1e-5 of max(|ref|, rms(ref)) on the parameter change, the moments and the norm), not its size."""
import numpy as np
import pytest
import torch

from oracle import adam as oadam
from tests.util import assert_close

pytestmark = pytest.mark.gpu

SIZES = [(1,), (3,), (4,), (4095,), (4096,), (4097,), (0,), (11,), (300, 333), (64, 1044)]


def run_steps(ver, sizes, steps, cfg_kw, clip):
    rng = np.random.default_rng(7)
    # small parameters: their fp32 resolution must stay below 1e-5 of the update
    p0 = [(0.01 * rng.standard_normal(s)).astype(np.float32) for s in sizes]
    cfg = ver.adam_cfg(max_grad_norm=clip, **cfg_kw)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    p = [dev(x) for x in p0]
    m = [torch.zeros_like(x) for x in p]
    v = [torch.zeros_like(x) for x in p]
    norm = torch.zeros(1, device="cuda")
    ws = ver.workspace(ver.ver_adam_workspace_bytes())
    rp, rm, rv = [x.astype(np.float64) for x in p0], [np.zeros(s) for s in sizes], [np.zeros(s) for s in sizes]
    for k in steps:
        grads = [(rng.standard_normal(s) * 10.0 ** rng.integers(-2, 2)).astype(np.float32) for s in sizes]
        before = [x.cpu().numpy().astype(np.float64) for x in p]
        ver.ver_adam_step(cfg, p, [dev(g) for g in grads], m, v, k, norm, ws)
        torch.cuda.synchronize()
        lr = oadam.cosine_lr(k, cfg_kw["total_steps"], float(np.float32(cfg_kw["lr0"])), float(np.float32(cfg_kw.get("lr_final", 0.0))))
        # the oracle continues from the device's fp32 state, so that every step is compared on its own
        rp = before
        # hyper-parameters as the fp32 values the C structure holds
        f32 = lambda x: float(np.float32(x))
        new_p, rm, rv, rnorm = oadam.adam_step(rp, grads, rm, rv, k + 1, lr, f32(cfg_kw.get("beta1", 0.9)),
                                               f32(cfg_kw.get("beta2", 0.999)), f32(cfg_kw.get("eps", 1e-8)), f32(clip))
        assert float(norm.item()) == pytest.approx(rnorm, rel=1e-5)
        for i, s in enumerate(sizes):
            if np.prod(s) == 0:
                continue
            assert_close(p[i].cpu().numpy().astype(np.float64) - before[i], new_p[i] - before[i], 1e-5, f"step {k} delta[{i}]")
            assert_close(m[i].cpu().numpy(), rm[i], 1e-5, f"step {k} m[{i}]")
            assert_close(v[i].cpu().numpy(), rv[i], 1e-5, f"step {k} v[{i}]")
        # moments of the oracle follow the device's fp32 values from here on (no drift between the two)
        rm = [x.cpu().numpy().astype(np.float64) for x in m]
        rv = [x.cpu().numpy().astype(np.float64) for x in v]


@pytest.mark.parametrize("clip", [0.0, 0.7, 1e9])
def test_steps_match_oracle(ver, clip):
    run_steps(ver, SIZES, [0, 1, 2, 50, 100, 130], dict(lr0=0.05, lr_final=0.002, total_steps=100), clip)


def test_paper_hyperparameters_first_and_last_step(ver):
    """Initial rate 2.5e-4 decayed to zero: the first step moves every parameter by about the rate, the step at
    the end of the schedule moves nothing."""
    x = torch.ones(5000, device="cuda")
    g = torch.full_like(x, 0.3)
    m, v = torch.zeros_like(x), torch.zeros_like(x)
    cfg = ver.adam_cfg(lr0=2.5e-4, lr_final=0.0, total_steps=10)
    ver.ver_adam_step(cfg, [x], [g], [m], [v], 0, None, None)
    torch.cuda.synchronize()
    assert torch.allclose(x, torch.full_like(x, 1.0 - 2.5e-4), atol=1e-7)
    y = x.clone()
    ver.ver_adam_step(cfg, [x], [g], [m], [v], 10, None, None)
    torch.cuda.synchronize()
    assert torch.equal(x, y)


def test_bitwise_reproducible_and_empty(ver):
    sizes = [(70000,), (123,), (0,)]
    outs = []
    for _ in range(2):
        p = [torch.from_numpy(np.random.default_rng(5).standard_normal(s).astype(np.float32)).cuda() for s in sizes]
        g = [torch.from_numpy(np.random.default_rng(6).standard_normal(s).astype(np.float32)).cuda() for s in sizes]
        m = [torch.zeros_like(x) for x in p]
        v = [torch.zeros_like(x) for x in p]
        norm = torch.zeros(1, device="cuda")
        ws = ver.workspace(ver.ver_adam_workspace_bytes())
        ver.ver_adam_step(ver.adam_cfg(lr0=0.01, total_steps=5, max_grad_norm=1.0), p, g, m, v, 1, norm, ws)
        torch.cuda.synchronize()
        outs.append([x.cpu().numpy() for x in p + m + v] + [norm.cpu().numpy()])
    assert all(np.array_equal(a, b) for a, b in zip(*outs))
    # nothing to do is not an error
    ver.ver_adam_step(ver.adam_cfg(total_steps=5), [], [], [], [], 0, None, None)


def test_bounded_step_projects_after_the_update(ver):
    """ver_adam_step_bounded: per-tensor boxes.  A tensor without bounds moves as in ver_adam_step; a bounded one
    is the oracle's step followed by the oracle's projection, bit-exact where the bound is hit."""
    rng = np.random.default_rng(3)
    sizes = [(5000,), (1,), (1,), (33,)]
    lower = [-np.inf, 1e-4, 1e-4, -0.004]
    upper = [np.inf, 1.0, 1.0, 0.004]
    p0 = [(0.01 * rng.standard_normal(s)).astype(np.float32) for s in sizes]
    p0[1][:] = 1.05e-4        # will be pushed below the lower bound
    p0[2][:] = 0.004          # stays inside (small, so that fp32 resolves the step to 1e-5)
    grads = [rng.standard_normal(s).astype(np.float32) for s in sizes]
    grads[1][:] = 3.0
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    cfg_kw = dict(lr0=1e-3, lr_final=0.0, total_steps=10)
    cfg = ver.adam_cfg(**cfg_kw)
    ws = ver.workspace(ver.ver_adam_workspace_bytes())
    p, q = [dev(x) for x in p0], [dev(x) for x in p0]
    mp, vp = [torch.zeros_like(x) for x in p], [torch.zeros_like(x) for x in p]
    mq, vq = [torch.zeros_like(x) for x in p], [torch.zeros_like(x) for x in p]
    g = [dev(x) for x in grads]
    ver.ver_adam_step_bounded(cfg, p, g, mp, vp, lower, upper, 0, None, ws)
    ver.ver_adam_step(cfg, q, g, mq, vq, 0, None, ws)
    torch.cuda.synchronize()
    f32 = lambda x: float(np.float32(x))
    new_p, _, _, _ = oadam.adam_step([x.astype(np.float64) for x in p0], grads, [np.zeros(s) for s in sizes],
                                     [np.zeros(s) for s in sizes], 1, f32(1e-3), f32(0.9), f32(0.999), f32(1e-8))
    want = oadam.project(new_p, [f32(x) for x in lower], [f32(x) for x in upper])
    assert torch.equal(p[0], q[0]) and torch.equal(p[2], q[2])            # no bound hit: same as the plain step
    assert p[1].item() == np.float32(1e-4) and q[1].item() < 1e-4         # clamped exactly to the bound
    got3 = p[3].cpu().numpy()
    assert got3.max() == np.float32(0.004) and got3.min() == np.float32(-0.004)
    hit = (want[3] == f32(0.004)) | (want[3] == f32(-0.004))
    assert hit.any() and (~hit).any()
    assert np.array_equal(np.abs(got3) == np.float32(0.004), hit)
    for i, s in enumerate(sizes):
        assert_close(p[i].cpu().numpy().astype(np.float64) - p0[i], want[i] - p0[i], 1e-5, f"delta[{i}]")
    for a, b in zip(mp + vp, mq + vq):
        assert torch.equal(a, b)                                          # the moments do not see the projection
