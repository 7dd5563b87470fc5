"""ver_gae_static (the entry point that allocates nothing: its scratch is a device array inside the library)
against ver_gae and the oracle, through the C ABI: two calls in a row, the second on a smaller input, so that
whatever the first call left in the shared array must not matter."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import gae as ogae
from paper_2210_05064_amd import workloads as wl
from tests.gpu_util import dev, host, run_gae
from tests.util import assert_close

pytestmark = pytest.mark.gpu

GAMMA, LAM = 0.99, 0.95


def _rollout(seed, n_envs, steps, p_done):
    rng = np.random.default_rng(seed)
    L = wl.apportion_steps(steps, rng.lognormal(0.0, 1.0, n_envs))
    off = np.concatenate([[0], np.cumsum(L)]).astype(np.int32)
    r = (0.1 * rng.standard_normal(steps)).astype(np.float32)
    v = rng.standard_normal(steps).astype(np.float32)
    d = (rng.random(steps) < p_done).astype(np.uint8)
    lv = rng.standard_normal(n_envs).astype(np.float32)
    return r, v, d, lv, off


def _static(ver, r, v, d, lv, off):
    """Raw call through ctypes: device pointers and sizes only."""
    S, N = len(r), len(off) - 1
    t = [dev(r), dev(v), dev(d), dev(lv), dev(off)]
    adv = torch.full((S,), float("nan"), device="cuda")
    ret = torch.full((S,), float("nan"), device="cuda")
    st = ver.lib.ver_gae_static(*[C.c_void_p(x.data_ptr()) for x in t], N, S, GAMMA, LAM,
                                C.c_void_p(adv.data_ptr()), C.c_void_p(ret.data_ptr()),
                                C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == 0, ver.ver_status_string(st)
    torch.cuda.synchronize()
    return host(adv), host(ret)


def test_static_scratch_matches_workspace_entry_point(ver):
    # first call: many tiles with a ragged tail and tiles batched per ticket; second call: fewer, smaller tiles,
    # which finds the first call's words in the array
    for seed, n_envs, steps, p_done in [(1, 3000, 5 * 2 ** 20 // 2 + 777, 1 / 200), (2, 40, 3 * 2048 + 5, 1 / 50)]:
        r, v, d, lv, off = _rollout(seed, n_envs, steps, p_done)
        adv_s, ret_s = _static(ver, r, v, d, lv, off)
        adv_w, ret_w = run_gae(ver, r, v, d, lv, off, GAMMA, LAM)
        assert_close(adv_s, adv_w, 1e-5, f"adv vs ver_gae, S={steps}")
        assert_close(ret_s, ret_w, 1e-5, f"ret vs ver_gae, S={steps}")
        adv_o, ret_o = ogae.gae(r, v, d, lv, off, GAMMA, LAM)
        assert_close(adv_s, adv_o, 1e-5, f"adv vs oracle, S={steps}")
        assert_close(ret_s, ret_o, 1e-5, f"ret vs oracle, S={steps}")


def test_static_scratch_rejects_what_does_not_fit(ver):
    S = (1 << 22) + 1
    z = torch.zeros(8, device="cuda")
    p = C.c_void_p(z.data_ptr())
    st = ver.lib.ver_gae_static(p, p, p, p, p, 1, S, GAMMA, LAM, p, p, None)   # rejected on the host: nothing is read
    assert st == -5 and "scratch" in ver.ver_status_string(st)
    assert ver.lib.ver_gae_static(p, p, p, p, p, 1, 0, GAMMA, LAM, p, p, None) == 0   # S = 0: no work
