"""The HBM-bound kernels far above the paper's sizes, where they change strategy: several tiles per ticket
in the advantage scan, several rounds per workgroup in the loss, the two-level counter scan and two
digit passes in the bucketing, windows of many environments in the importance weights.  The oracle is
called on sampled environments / on the whole input where it finishes in seconds; exact closed forms
cover what it cannot reach."""
import numpy as np
import pytest
import torch

from oracle.gae import gae as oracle_gae
from oracle.ingest import ingest as oracle_ingest
from oracle.is_weight import is_weights as oracle_is_weights
from oracle.ppo_loss import ppo_loss as oracle_ppo_loss
from paper_2210_05064_amd import workloads as wl
from tests.gpu_util import dev, host, run_gae
from tests.util import assert_close

pytestmark = pytest.mark.gpu
GAE_TILE = 2048


def _ragged(n_envs, budget, seed, empty_every=0):
    rng = np.random.default_rng(seed)
    L = wl.apportion_steps(budget, rng.lognormal(0.0, 1.0, size=n_envs)).astype(np.int64)
    if empty_every:                      # move some environments' steps to their neighbour: empty stretches
        idx = np.arange(empty_every, n_envs, empty_every)
        L[idx - 1] += L[idx]
        L[idx] = 0
    off = np.zeros(n_envs + 1, np.int32)
    off[1:] = np.cumsum(L)
    return rng, off


@pytest.mark.parametrize("S,N,aligned", [(1 << 24, 1 << 17, True), ((1 << 22) + 4099, 30000, True),
                                          ((1 << 22) + 6, 30000, False), ((1 << 27) + 1000, 1 << 20, True)])
def test_gae_many_tiles_sampled_environments(ver, S, N, aligned):
    """8192 (or 2049, or 65537) tiles: several tiles share a ticket (8, 2, and the maximum of 64).  Environments are
    independent, so the oracle recomputes sampled ones: random ones and those that contain a tile boundary next
    to a batch boundary."""
    rng, off = _ragged(N, S, seed=S % 1000, empty_every=97)
    r = (0.1 * rng.standard_normal(S)).astype(np.float32)
    v = rng.standard_normal(S).astype(np.float32)
    d = (rng.random(S) < 1.0 / 200).astype(np.uint8)
    lv = rng.standard_normal(N).astype(np.float32)
    if aligned:
        adv, ret = run_gae(ver, r, v, d, lv, off, 0.99, 0.95)
    else:   # arrays that start 4 bytes (1 byte for dones) past an aligned address: the element-wise path
        pad = lambda a: dev(np.concatenate([a[:1], a]))[1:]
        r_t, v_t, d_t, lv_t, off_t = pad(r), pad(v), pad(d), dev(lv), dev(off)
        adv_t, ret_t = torch.empty(S + 1, device="cuda")[1:], torch.empty(S + 1, device="cuda")[1:]
        ws = ver.workspace(ver.ver_gae_workspace_bytes(S))
        ver.lib.ver_gae(r_t.data_ptr(), v_t.data_ptr(), d_t.data_ptr(), lv_t.data_ptr(), off_t.data_ptr(),
                        N, S, 0.99, 0.95, adv_t.data_ptr(), ret_t.data_ptr(), ws.data_ptr(), ws.numel() * 4,
                        torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert ws[1].item() == 0
        adv, ret = host(adv_t), host(ret_t)
    ntiles = (S + GAE_TILE - 1) // GAE_TILE
    edges = [(ntiles - 1 - t) * GAE_TILE for t in range(0, ntiles, max(1, ntiles // 64))]   # first step of a tile
    envs = set(rng.integers(0, N, size=150).tolist())
    envs |= {int(np.searchsorted(off, k, side="right") - 1) for k in edges if 0 < k < S}
    g, lam = np.float32(0.99).item(), np.float32(0.95).item()
    for e in sorted(envs):
        a, b = int(off[e]), int(off[e + 1])
        if a == b:
            continue
        a_ref, r_ref = oracle_gae(r[a:b], v[a:b], d[a:b], lv[e:e + 1], np.array([0, b - a]), g, lam)
        assert_close(adv[a:b], a_ref, 1e-5, f"adv of environment {e}")
        assert_close(ret[a:b], r_ref, 1e-5, f"ret of environment {e}")
    assert np.isfinite(adv).all() and np.isfinite(ret).all()


def test_gae_carry_through_every_tile_and_batch(ver):
    """One environment of 2^23 steps, no episode end, gamma = lambda = 1, reward 1, value 0: the advantage of
    step k is the number of steps left plus the bootstrap value, exactly (integers below 2^24); every tile's
    map has a = 1, so the chain of published maps runs through all 4096 tiles and all tickets."""
    S = 1 << 23
    r, v, d = np.ones(S, np.float32), np.zeros(S, np.float32), np.zeros(S, np.uint8)
    adv, ret = run_gae(ver, r, v, d, np.array([5.0], np.float32), np.array([0, S], np.int32), 1.0, 1.0)
    expect = (S - np.arange(S) + 5).astype(np.float32)
    assert np.array_equal(adv, expect)
    assert np.array_equal(ret, expect)


@pytest.mark.parametrize("S,N", [(1 << 22, 1 << 15), ((1 << 25) + 5, 1 << 18)])
def test_is_weight_many_environments(ver, S, N):
    """The larger case gives a workgroup several consecutive tiles (offsets of a tile taken from next to the
    tile before)."""
    _, off = _ragged(N, S, seed=5, empty_every=50)
    w = torch.empty(S, device="cuda")
    ver.ver_is_weight(dev(off), N, S, 1.0, w)
    ref = oracle_is_weights(off, 1.0).astype(np.float32)
    assert np.array_equal(host(w), ref)
    # windows of more environments than a workgroup keeps in LDS, and more than the near window holds: thousands
    # of empty environments in a row, in the middle of a tile and across tile boundaries
    off2 = np.concatenate([[0], np.full(6000, 3000), [S // 2] * 5000, np.full(700, S // 2 + 4096 * 3 + 17),
                           np.arange(S // 2 + 4096 * 3 + 18, S // 2 + 4096 * 3 + 18 + 3000), [S]]).astype(np.int32)
    N2 = len(off2) - 1
    ver.ver_is_weight(dev(off2), N2, S, 4.0, w)
    assert np.array_equal(host(w), oracle_is_weights(off2, 4.0).astype(np.float32))


BIG = 2048 * 256 + 3 * 256 + 77   # more rows than one sweep of the grid covers (2048 workgroups x 256 rows)


@pytest.mark.parametrize("dist,A,shift,M", [(1, 11, 0, BIG), (0, 4, 1, BIG), (1, 20, 0, BIG), (1, 11, 1, 5000),
                                             (0, 4, 0, 5000), (1, 11, 0, BIG - 1), (0, 4, 0, BIG), (1, 6, 0, BIG + 1),
                                             (1, 16, 0, 70001), (0, 3, 0, 40004), (1, 1, 0, 12)])
def test_loss_several_rounds_per_workgroup(ver, dist, A, shift, M):
    """Several blocks per workgroup and a ragged last block; shift = 1: row arrays that start 4 bytes past a
    16-byte boundary (the word-by-word copies).  Aligned arrays with M * A a multiple of 4 and A <= 16 take the
    kernel specialised on the row width (BIG - 1 rows of 11, BIG of 4, BIG + 1 of 6, 70001 of 16, 40004 of 3, 12 of
    1), every other case the general one."""
    rng = np.random.default_rng(40 + A)
    u = rng.standard_normal((M, A)).astype(np.float32)
    value, ret, adv = (rng.standard_normal(M).astype(np.float32) for _ in range(3))
    isw = rng.random(M).astype(np.float32)
    if dist == 1:
        acts = rng.standard_normal((M, A)).astype(np.float32)
        log_std = (0.1 * rng.standard_normal(A)).astype(np.float32)
    else:
        acts = rng.integers(0, A, size=M).astype(np.int32)
        log_std = None
    # old log-probabilities near the new ones, so that ratios stay around 1 and some rows are clipped
    if dist == 1:
        z = (acts - u) * np.exp(-log_std)
        logp = (-0.5 * z * z - log_std - 0.5 * np.log(2 * np.pi)).sum(1)
    else:
        lse = np.log(np.exp(u - u.max(1, keepdims=True)).sum(1)) + u.max(1)
        logp = u[np.arange(M), acts] - lse
    noise = 0.15 * rng.standard_normal(M)
    # which side of the clip a row falls on is decided in fp32 on the GPU and in fp64 by the oracle: keep every
    # ratio away from the two boundaries, where the two could legitimately disagree
    rho = np.exp(-noise)
    noise[(np.abs(rho - 0.8) < 2e-3) | (np.abs(rho - 1.2) < 2e-3)] = 0.0
    logp_old = (logp + noise).astype(np.float32)
    f32 = dict(dtype=torch.float32, device="cuda")
    def rows(a):   # [M, A] device copy, optionally starting one element past an aligned address
        t = torch.empty(M * A + shift, dtype=torch.from_numpy(a[:1]).dtype, device="cuda")[shift:].view(M, A)
        t.copy_(torch.from_numpy(a))
        return t
    scalars, d_v = torch.zeros(6, **f32), torch.empty(M, **f32)
    d_u = torch.empty(M * A + shift, **f32)[shift:].view(M, A)
    d_ls = torch.empty(A, **f32)
    ws = ver.workspace(ver.ver_ppo_loss_workspace_bytes(M, A))
    ver.ver_ppo_loss(ver.ppo_cfg(0.2, 0.5, 1e-2, dist, A), M, rows(u), dev(value), dev(log_std) if dist == 1 else None,
                     rows(acts) if dist == 1 else dev(acts), dev(logp_old), dev(adv), dev(ret), dev(isw), scalars, d_u,
                     d_v, d_ls if dist == 1 else None, ws)
    r_scalars, r_du, r_dv, r_dls = oracle_ppo_loss(dist, u, value, log_std, acts, logp_old, adv, ret, 0.2, 0.5, 1e-2,
                                                   weight=isw)
    names = ["total", "policy", "value", "entropy", "approx_kl", "clip_frac"]
    got = host(scalars)
    for i, n in enumerate(names):
        assert abs(got[i] - r_scalars[n]) <= 1e-4 * max(1.0, abs(r_scalars[n])), (n, got[i], r_scalars[n])
    assert_close(host(d_u), r_du, 1e-4, "d_head_out")
    assert_close(host(d_v), r_dv, 1e-4, "d_value")
    if dist == 1:
        assert_close(host(d_ls), r_dls, 1e-4, "d_log_std")


def test_ingest_two_passes_two_level_scan(ver):
    """2^22 slots of 40000 environments: two digit passes, counters scanned by many workgroups; a few ids
    outside [0, N) as well."""
    S, N = 1 << 22, 40000
    _, off = _ragged(N, S, seed=9, empty_every=61)
    arr_env, arr_t, _ = wl.arrival_order(off, seed=10)
    arr_env = arr_env.copy()
    bad = np.random.default_rng(11).choice(S, 5, replace=False)
    arr_env[bad] = [-1, N, N + 7, 2 ** 31 - 1, -2 ** 31]
    i32 = dict(dtype=torch.int32, device="cuda")
    env_off, order, info = torch.empty(N + 1, **i32), torch.empty(S, **i32), torch.empty(4, **i32)
    ws = ver.workspace(ver.ver_ingest_workspace_bytes(N, S))
    ws.fill_(-1)
    arr_t = arr_t.copy()
    arr_t[np.random.default_rng(12).choice(S, 6, replace=False)] -= 2
    ver.ver_ingest(dev(arr_env), dev(arr_t), N, S, env_off, order, info, ws)
    good = np.flatnonzero((arr_env >= 0) & (arr_env < N))
    ref_off, ref_order, ref_viol = oracle_ingest(arr_env[good], N, arr_t[good])
    assert np.array_equal(host(env_off), ref_off)
    n_good = len(good)
    assert np.array_equal(host(order)[:n_good], good[ref_order])
    assert ref_viol > 0 and host(info).tolist() == [ref_viol, len(bad), 0, 0]
    assert host(order)[n_good:].tolist() == sorted(bad.tolist())


def test_ingest_large_buffer_one_pass_with_counter_check(ver):
    """2^20 + 777 slots of 300 environments (one digit pass, tiles that leave through LDS in sorted order, ragged
    last tile), with the per-environment step counters checked and a few of them broken on purpose."""
    S, N = (1 << 20) + 777, 300
    _, off = _ragged(N, S, seed=21, empty_every=7)
    arr_env, arr_t, _ = wl.arrival_order(off, seed=22)
    arr_t = arr_t.copy()
    arr_t[np.random.default_rng(23).choice(S, 9, replace=False)] += 3
    i32 = dict(dtype=torch.int32, device="cuda")
    env_off, order, info = torch.empty(N + 1, **i32), torch.empty(S, **i32), torch.empty(4, **i32)
    ws = ver.workspace(ver.ver_ingest_workspace_bytes(N, S))
    ws.fill_(-1)
    ver.ver_ingest(dev(arr_env), dev(arr_t), N, S, env_off, order, info, ws)
    ref_off, ref_order, ref_bad = oracle_ingest(arr_env, N, arr_t)
    assert np.array_equal(host(env_off), ref_off)
    assert np.array_equal(host(order), ref_order)
    assert ref_bad > 0 and host(info).tolist() == [ref_bad, 0, 0, 0]


def test_ingest_at_its_size_limit(ver):
    """2^24 slots is the most one call takes (511 environments: one 9-bit pass); one more is refused."""
    S, N = 1 << 24, 511
    rng = np.random.default_rng(31)
    arr_env = rng.integers(0, N, size=S).astype(np.int32)
    i32 = dict(dtype=torch.int32, device="cuda")
    env_off, order, info = torch.empty(N + 1, **i32), torch.empty(S, **i32), torch.empty(4, **i32)
    ws = ver.workspace(ver.ver_ingest_workspace_bytes(N, S))
    ver.ver_ingest(dev(arr_env), None, N, S, env_off, order, info, ws)
    ref_off, ref_order, _ = oracle_ingest(arr_env, N)
    assert np.array_equal(host(env_off), ref_off)
    assert np.array_equal(host(order), ref_order)
    assert host(info).tolist() == [0, 0, 0, 0]
    assert ver.ver_ingest_workspace_bytes(N, S + 1) == 0
    with pytest.raises(ver.VerError) as e:
        ver.ver_ingest(dev(arr_env), None, N, S + 1, env_off, order, info, ws)
    assert e.value.status == -3
