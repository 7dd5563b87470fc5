"""ver_ppo_loss against the CPU oracle.  Tolerance 1e-4 relative per tensor."""
import numpy as np
import pytest
import torch

from oracle import ppo_loss as opl
from tests.gpu_util import dev, host
from tests.util import assert_close

pytestmark = pytest.mark.gpu
TOL = 1e-4
NAMES = ["total", "policy", "value", "entropy", "approx_kl", "clip_frac"]


def make(rng, dist, M, A):
    u = rng.standard_normal((M, A)).astype(np.float32)
    v = rng.standard_normal(M).astype(np.float32)
    ls = (0.3 * rng.standard_normal(A)).astype(np.float32) if dist == 1 else None
    act = rng.integers(0, A, M).astype(np.int32) if dist == 0 else rng.standard_normal((M, A)).astype(np.float32)
    logp = np.array([opl.row_logp_entropy(dist, u[p].astype(np.float64), act[p], None if ls is None else ls.astype(np.float64))[0]
                     for p in range(M)])
    logp_old = (logp + 0.1 * rng.standard_normal(M)).astype(np.float32)
    return dict(u=u, v=v, ls=ls, act=act, logp_old=logp_old, adv=rng.standard_normal(M).astype(np.float32),
                ret=rng.standard_normal(M).astype(np.float32))


def run(ver, dist, x, clip=0.2, cv=0.5, ce=1e-2, weight=None):
    M, A = x["u"].shape
    cfg = ver.ppo_cfg(clip, cv, ce, dist, A)
    scal = torch.full((6,), float("nan"), device="cuda")
    d_u = torch.full((M, A), float("nan"), device="cuda")
    d_v = torch.full((M,), float("nan"), device="cuda")
    d_ls = torch.full((A,), float("nan"), device="cuda")
    ws = ver.workspace(ver.ver_ppo_loss_workspace_bytes(M, A))
    ws.fill_(-1)
    ver.ver_ppo_loss(cfg, M, dev(x["u"]), dev(x["v"]), dev(x["ls"]) if dist == 1 else None, dev(x["act"]),
                     dev(x["logp_old"]), dev(x["adv"]), dev(x["ret"]), dev(weight) if weight is not None else None,
                     scal, d_u, d_v, d_ls, ws)
    torch.cuda.synchronize()
    return host(scal), host(d_u), host(d_v), host(d_ls)


def check(ver, dist, x, ce=1e-2, weight=None):
    scal, d_u, d_v, d_ls = run(ver, dist, x, ce=ce, weight=weight)
    f32 = lambda c: float(np.float32(c))
    ref, r_u, r_v, r_ls = opl.ppo_loss(dist, x["u"], x["v"], x["ls"], x["act"], x["logp_old"], x["adv"], x["ret"],
                                       f32(0.2), 0.5, f32(ce), weight)
    for i, n in enumerate(NAMES):
        if n == "clip_frac":
            # a row whose ratio sits within rounding of the clip edge may flip; allow one row
            assert abs(scal[i] - ref[n]) <= 1.5 / len(x["v"]), (scal[i], ref[n])
        else:
            assert abs(scal[i] - ref[n]) <= TOL * max(abs(ref[n]), 1e-2), (n, scal[i], ref[n])
    assert_close(d_u, r_u, TOL, "d_head_out")
    assert_close(d_v, r_v, TOL, "d_value")
    if dist == 1:
        assert_close(d_ls, r_ls, TOL, "d_log_std")


@pytest.mark.parametrize("dist,A,M", [(0, 4, 64), (0, 4, 1024), (0, 4, 8192), (1, 11, 1024), (1, 11, 8192),
                                      (0, 7, 777), (1, 3, 1), (0, 2, 300001), (1, 11, 300001)])
def test_against_oracle(ver, dist, A, M):
    """Workload sizes (64 ... 8192 rows), ragged sizes, one row, and a size that
    needs several rounds per workgroup."""
    rng = np.random.default_rng(M + A)
    if M > 100000:           # oracle is a Python row loop: check a bounded prefix through the weights
        x = make(rng, dist, 4096, A)
        big = {k: (np.concatenate([v] * 74)[:M] if v is not None and k != "ls" else v) for k, v in x.items()}
        w = np.zeros(M, np.float32)
        w[:4096] = M / 4096.0          # rows beyond the prefix carry weight 0
        scal, d_u, d_v, d_ls = run(ver, dist, big, weight=w)
        ref, r_u, r_v, r_ls = opl.ppo_loss(dist, x["u"], x["v"], x["ls"], x["act"], x["logp_old"], x["adv"],
                                           x["ret"], float(np.float32(0.2)), 0.5, float(np.float32(1e-2)))
        for i, n in enumerate(NAMES[:4]):
            assert abs(scal[i] - ref[n]) <= TOL * max(abs(ref[n]), 1e-2), (n, scal[i], ref[n])
        assert_close(d_u[:4096], r_u, TOL, "d_head_out")
        assert np.all(d_u[4096:] == 0) and np.all(d_v[4096:] == 0)
        if dist == 1:
            assert_close(d_ls, r_ls, TOL, "d_log_std")
        return
    check(ver, dist, make(rng, dist, M, A))


@pytest.mark.parametrize("dist,A", [(0, 4), (1, 11)])
def test_row_weights(ver, dist, A):
    rng = np.random.default_rng(3)
    x = make(rng, dist, 500, A)
    check(ver, dist, x, weight=rng.random(500).astype(np.float32))


@pytest.mark.parametrize("dist,A", [(0, 4), (1, 11)])
def test_invariants_on_device(ver, dist, A):
    """ratio = 1: policy loss = -mean(adv), nothing clipped; zero advantages:
    no policy gradient (entropy coefficient 0)."""
    rng = np.random.default_rng(4)
    x = make(rng, dist, 999, A)
    # logp_old = the device's own logp: obtained from approx_kl-free route: use oracle logp rounded to fp32
    x0 = dict(x)
    x0["adv"] = np.zeros_like(x["adv"])
    scal, d_u, _, d_ls = run(ver, dist, x0, ce=0.0)
    assert scal[1] == 0 and np.all(d_u == 0)
    if dist == 1:
        assert np.all(d_ls == 0)


def test_reproducible_and_errors(ver):
    rng = np.random.default_rng(5)
    x = make(rng, 1, 5000, 11)
    a, b = run(ver, 1, x), run(ver, 1, x)
    assert all(np.array_equal(p, q) for p, q in zip(a, b))
    with pytest.raises(ver.VerError):
        cfg = ver.ppo_cfg(0.2, 0.5, 0.0, 0, 64)
        t = torch.zeros(64, device="cuda")
        ver.ver_ppo_loss(cfg, 1, t, t, None, t.to(torch.int32), t, t, t, None, t, t, t, None, ver.workspace(4096))


@pytest.mark.parametrize("dist,A,M", [(0, 4, 1024), (1, 11, 8192), (0, 7, 777), (1, 3, 1)])
@pytest.mark.parametrize("alpha,target,sign", [(1e-3, 0.0, 1.0), (0.35, 1.5, -1.0)])
def test_learned_entropy_coefficient(ver, dist, A, M, alpha, target, sign):
    """ver_ppo_loss_learned_entropy against the oracle: the coefficient comes from device memory, the total
    carries alpha's own term, d_alpha = sign * (target - H); the policy's gradients are those at c_e = alpha."""
    from oracle import entropy_coef as oec
    rng = np.random.default_rng(M + A)
    x = make(rng, dist, M, A)
    weight = rng.random(M).astype(np.float32) if M > 1 else None
    cfg = ver.ppo_cfg(0.2, 0.5, 123.0, dist, A)          # the fixed coefficient must be ignored
    scal = torch.full((6,), float("nan"), device="cuda")
    d_u = torch.full((M, A), float("nan"), device="cuda")
    d_v = torch.full((M,), float("nan"), device="cuda")
    d_ls = torch.full((A,), float("nan"), device="cuda")
    d_alpha = torch.full((1,), float("nan"), device="cuda")
    a_dev = torch.tensor([alpha], dtype=torch.float32, device="cuda")
    ws = ver.workspace(ver.ver_ppo_loss_workspace_bytes(M, A))
    ws.fill_(-1)
    ver.ver_ppo_loss_learned_entropy(cfg, M, dev(x["u"]), dev(x["v"]), dev(x["ls"]) if dist == 1 else None, dev(x["act"]),
                                     dev(x["logp_old"]), dev(x["adv"]), dev(x["ret"]),
                                     dev(weight) if weight is not None else None, a_dev, target, sign,
                                     scal, d_u, d_v, d_ls, d_alpha, ws)
    torch.cuda.synchronize()
    f32 = lambda c: float(np.float32(c))
    ref, r_u, r_v, r_ls, r_alpha = oec.ppo_loss_learned_entropy(
        dist, x["u"], x["v"], x["ls"], x["act"], x["logp_old"], x["adv"], x["ret"], f32(0.2), 0.5, f32(alpha),
        f32(target), weight, sign)
    scal = host(scal)
    for i, n in enumerate(NAMES[:5]):
        assert abs(scal[i] - ref[n]) <= TOL * max(abs(ref[n]), 1e-2), (n, scal[i], ref[n])
    assert abs(host(d_alpha)[0] - r_alpha) <= TOL * max(abs(r_alpha), 1e-2)
    assert host(a_dev)[0] == np.float32(alpha)           # read only
    assert_close(host(d_u), r_u, TOL, "d_head_out")
    assert_close(host(d_v), r_v, TOL, "d_value")
    if dist == 1:
        assert_close(host(d_ls), r_ls, TOL, "d_log_std")
