"""End-to-end learner update through the C ABI against the CPU oracle chain
(GAE -> pack -> LSTM forward -> PPO loss -> LSTM backward), every minibatch."""
import numpy as np
import pytest
import torch

from oracle import gae as ogae, is_weight as ois, learner as olearner, pack as opack
from paper_2210_05064_amd import workloads as wl
from tests.gpu_util import GRAD_NAMES, grads_to_list, host
from tests.util import assert_close, assert_close_update, closer

pytestmark = pytest.mark.gpu


def run_case(w, seed, compute=None, max_is=None, arrival=False):
    from paper_2210_05064_amd.learner import Learner
    ro = wl.make_rollout(w, seed=seed, bias_scale=0.1)
    adv, ret = ogae.gae(ro["rewards"], ro["values"], ro["dones"], ro["last_values"], ro["env_off"], w.gamma, w.lam)
    logp_old = (olearner.collection_logp(ro, ro["weights"], ro["dones"], ro["env_off"], w.dist,
                                         ro["env_started_episode"], ro["rnn_h"], ro["rnn_c"])
                + ro["logp_noise"]).astype(np.float32)
    arr = wl.arrival_order(ro["env_off"], seed=seed + 100, t_start=np.arange(ro["N"])) if arrival else None
    L = Learner(ro, compute=compute, want_dx=True, max_is=max_is, arrival=arr)
    weight = None if max_is is None else ois.is_weights(ro["env_off"], max_is)
    L.set_logp_old(torch.from_numpy(logp_old).cuda())
    if arrival:
        assert int(L.env_off.abs().sum().item()) == 0 and float(L.obs.abs().sum().item()) == 0.0   # nothing environment-major yet
    cfg = dict(dist=w.dist, clip=np.float32(w.clip).item(), value_coef=w.value_coef,
               entropy_coef=np.float32(w.entropy_coef).item())
    names = [f"layer{l}.{n}" for l in range(w.n_layers) for n in GRAD_NAMES] + ["W_a", "b_a", "w_v", "b_v"]
    close = closer(L.compute)
    checked = []

    def check(e, b):
        torch.cuda.synchronize()
        assert not L.lstm_timed_out()
        meta = opack.pack_minibatch(ro["dones"], ro["env_off"], ro["seq_key"][e], L.B, b, ro["env_started_episode"])
        assert np.array_equal(host(L.gather_idx), meta["gather_idx"])
        assert host(L.info).tolist()[:3] == [meta["n_seq"], meta["T_max"], meta["K"]]
        h0 = opack.initial_states(ro["rnn_h"], meta["seq_first"], meta["seq_is_ep_start"])
        c0 = opack.initial_states(ro["rnn_c"], meta["seq_first"], meta["seq_is_ep_start"])
        ref = olearner.minibatch_step(ro, ro["weights"], meta, cfg, adv, ret, logp_old, h0, c0, weight=weight, want_dx=True)
        close(host(L.head_out), ref["u"], "head_out")
        close(host(L.value), ref["v"], "value")
        sc = host(L.scalars)
        for i, n in enumerate(["total", "policy", "value", "entropy", "approx_kl"]):
            tol = 1e-4 if L.compute == 0 else 2e-2
            assert abs(sc[i] - ref["scalars"][n]) <= tol * max(abs(ref["scalars"][n]), 1e-2), (n, sc[i], ref["scalars"][n])
        assert abs(sc[5] - ref["scalars"]["clip_frac"]) <= (1.5 if L.compute == 0 else 0.02 * L.M + 1.5) / L.M
        close(host(L.d_head), ref["d_u"], "d_head_out")
        close(host(L.d_x), ref["d_x"], "d_x")
        for n, g, r in zip(names, L.grads, grads_to_list(ref["grads"])):
            close(host(g), r, n)
        if w.dist == 1:
            close(host(L.d_log_std), ref["grads"]["log_std"], "d_log_std")
        checked.append((e, b))

    L.update(on_minibatch=check)
    assert_close(host(L.adv), adv, 1e-5, "adv")
    assert_close(host(L.ret), ret, 1e-5, "ret")
    assert len(checked) == w.epochs * L.B
    if arrival:
        assert np.array_equal(host(L.env_off), ro["env_off"]) and host(L.ingest_info).tolist() == [0, 0, 0, 0]
        assert np.array_equal(host(L.obs), ro["obs"]) and np.array_equal(host(L.rnn_c), ro["rnn_c"])


def test_tiny_workload_update(ver):
    run_case(wl.WORKLOADS["tiny"], seed=1)


@pytest.mark.parametrize("name", ["tiny", "manip", "large"])
def test_update_from_the_arrival_order_buffer(ver, name):
    """The rollout handed over as the linear collection buffer (steps interleaved across environments): the
    update buckets it by environment on the GPU first; everything downstream against the oracle chain on the
    environment-major rollout."""
    w = wl.WORKLOADS[name]
    if name != "tiny":
        w = wl.scaled(w, budget=w.budget // 8, n_envs=w.n_envs // 2, hidden=128, input_dim=w.input_dim // 16 * 4, epochs=1)
    run_case(w, seed=8, compute=0, max_is=1.0, arrival=True)


@pytest.mark.parametrize("name,max_is", [("tiny", 1.0), ("manip", 1.0), ("nav", 1.5)])
def test_update_with_importance_weights(ver, name, max_is):
    """The per-step truncated importance weight computed, packed and applied in the loss on the GPU: every
    minibatch's loss scalars and gradients against the oracle chain given the oracle's weights."""
    w = wl.WORKLOADS[name]
    if name != "tiny":
        w = wl.scaled(w, budget=w.budget // 4, n_envs=w.n_envs // 2, hidden=128, input_dim=w.input_dim // 16 * 4, epochs=1)
    run_case(w, seed=5, compute=0, max_is=max_is)


@pytest.mark.parametrize("name,compute", [("nav", 0), ("manip", 0), ("large", 1), ("max", 1)])
def test_workload_shaped_update_reduced_width(ver, name, compute):
    """The workload's ragged structure (envs, lengths, dones, epochs x
    minibatches, policy type) with a narrower network so that the oracle
    finishes in seconds."""
    w = wl.WORKLOADS[name]
    scale = 4 if name in ("nav", "manip") else 16
    w = wl.scaled(w, budget=w.budget // scale, n_envs=max(4, w.n_envs // scale), hidden=128, input_dim=w.input_dim // 4 // 4 * 4,
                  epochs=1)
    run_case(w, seed=2, compute=compute)


@pytest.mark.parametrize("dist,clip_norm,max_is", [(1, 0.0, None), (0, 0.5, None), (1, 0.5, 1.0)])
def test_update_with_optimizer(ver, dist, clip_norm, max_is):
    """A whole update with the Adam step in the loop (2 epochs x 2 minibatches = 4 optimiser steps), fp32 path:
    the weights after the update against the oracle chain.  Compared is the CHANGE of every tensor, relative to
    its own scale (the step size is ~lr, far below the size of the weights)."""
    from paper_2210_05064_amd.learner import Learner
    base = wl.WORKLOADS["manip" if dist == 1 else "nav"]
    w = wl.scaled(base, budget=384, n_envs=10, hidden=64, input_dim=20, p_done=0.03, epochs=2, minibatches=2)
    ro = wl.make_rollout(w, seed=41, bias_scale=0.1)
    adv, ret = ogae.gae(ro["rewards"], ro["values"], ro["dones"], ro["last_values"], ro["env_off"], w.gamma, w.lam)
    logp_old = (olearner.collection_logp(ro, ro["weights"], ro["dones"], ro["env_off"], w.dist,
                                         ro["env_started_episode"], ro["rnn_h"], ro["rnn_c"])
                + ro["logp_noise"]).astype(np.float32)
    opt = dict(lr0=2.5e-4, lr_final=0.0, total_steps=6, beta1=0.9, beta2=0.999, eps=1e-8, max_grad_norm=clip_norm)
    L = Learner(ro, compute=0, adam_total_steps=opt["total_steps"],
                adam={k: v for k, v in opt.items() if k != "total_steps"}, max_is=max_is, want_grad_norm=True)
    L.logp_old.copy_(torch.from_numpy(logp_old).cuda())
    before = [host(t).astype(np.float64) for t in L.opt_params]
    L.update()
    torch.cuda.synchronize()
    assert not L.lstm_timed_out() and L.opt_steps == 4
    f32 = lambda x: float(np.float32(x))
    cfg = dict(dist=w.dist, clip=f32(w.clip), value_coef=w.value_coef, entropy_coef=f32(w.entropy_coef),
               epochs=w.epochs, minibatches=w.minibatches)
    opt32 = {k: (f32(v) if k != "total_steps" else v) for k, v in opt.items()}
    ref_w, ref_scalars, ref_norms = olearner.ppo_update(ro, adv.astype(np.float32), ret.astype(np.float32), logp_old, cfg, opt32,
                                                        max_is=max_is)
    ref = olearner._flatten(ref_w, w.dist == 1)
    assert len(ref) == len(L.opt_params)
    assert float(L.grad_norm.item()) == pytest.approx(ref_norms[-1], rel=1e-3)
    for i, (t, b0, r) in enumerate(zip(L.opt_params, before, ref)):
        got = host(t).astype(np.float64) - b0
        want = r - b0
        assert np.max(np.abs(want)) > 1e-5, "the update must have moved the tensor"
        assert_close_update(got, want, f"change of tensor {i}")
    sc = host(L.scalars)
    assert abs(sc[0] - ref_scalars[-1]["total"]) <= 1e-3 * max(abs(ref_scalars[-1]["total"]), 1e-2)


@pytest.mark.parametrize("dist,sign,max_is", [(1, 1.0, None), (1, -1.0, 1.0), (0, -1.0, None)])
def test_update_with_learned_entropy_coefficient(ver, dist, sign, max_is):
    """The learned entropy coefficient in the loop (2 epochs x 2 minibatches): it lives in device memory, the loss
    reads it and hands its gradient to the optimiser, which keeps it inside its bounds.  Its trajectory (bounds
    tight enough to be hit), the weights and the last minibatch's loss against the oracle chain."""
    from paper_2210_05064_amd.learner import Learner
    base = wl.WORKLOADS["manip" if dist == 1 else "nav"]
    w = wl.scaled(base, budget=384, n_envs=10, hidden=64, input_dim=20, p_done=0.03, epochs=2, minibatches=2)
    ro = wl.make_rollout(w, seed=43, bias_scale=0.1)
    adv, ret = ogae.gae(ro["rewards"], ro["values"], ro["dones"], ro["last_values"], ro["env_off"], w.gamma, w.lam)
    logp_old = (olearner.collection_logp(ro, ro["weights"], ro["dones"], ro["env_off"], w.dist,
                                         ro["env_started_episode"], ro["rnn_h"], ro["rnn_c"])
                + ro["logp_noise"]).astype(np.float32)
    f32 = lambda x: float(np.float32(x))
    opt = dict(lr0=2.5e-4, lr_final=0.0, total_steps=6, beta1=0.9, beta2=0.999, eps=1e-8, max_grad_norm=0.0)
    le = dict(alpha0=f32(1e-3), lower=f32(6e-4), upper=f32(1.4e-3))       # two steps of 2.5e-4 leave the box
    L = Learner(ro, compute=0, adam_total_steps=opt["total_steps"],
                adam={k: v for k, v in opt.items() if k != "total_steps"}, max_is=max_is,
                learned_entropy=dict(le, target=0.0, sign=sign))
    L.logp_old.copy_(torch.from_numpy(logp_old).cuda())
    before = [host(t).astype(np.float64) for t in L.opt_params]
    alphas = []
    L.update(on_minibatch=lambda e, b: alphas.append(float(L.alpha.item())))
    torch.cuda.synchronize()
    assert not L.lstm_timed_out() and L.opt_steps == 4
    cfg = dict(dist=w.dist, clip=f32(w.clip), value_coef=w.value_coef, target_entropy=0.0, alpha_sign=sign,
               epochs=w.epochs, minibatches=w.minibatches)
    opt32 = {k: (f32(v) if k != "total_steps" else v) for k, v in opt.items()}
    ref_w, ref_scalars, _, ref_alpha = olearner.ppo_update(ro, adv.astype(np.float32), ret.astype(np.float32), logp_old,
                                                           cfg, opt32, max_is=max_is, learned_entropy=le)
    assert alphas[-1] == pytest.approx(ref_alpha, rel=1e-4)
    assert le["lower"] <= min(alphas) and max(alphas) <= le["upper"]
    assert alphas[-1] in (np.float32(le["lower"]), np.float32(le["upper"])), "the bound must have been reached"
    assert abs(alphas[0] - le["alpha0"]) == pytest.approx(2.5e-4, rel=1e-3)     # Adam's first step: lr * sign
    ref = olearner._flatten(ref_w, w.dist == 1)
    for i, (t, b0, r) in enumerate(zip(L.opt_params[:-1], before, ref)):
        assert_close_update(host(t).astype(np.float64) - b0, r - b0, f"change of tensor {i}")
    sc = host(L.scalars)
    assert abs(sc[0] - ref_scalars[-1]["total"]) <= 1e-3 * max(abs(ref_scalars[-1]["total"]), 1e-2)


@pytest.mark.parametrize("name,compute", [("manip", 0), ("large", 1)])
def test_whole_update_is_bitwise_reproducible(ver, name, compute):
    """Two learners built from the same rollout run two updates each (arrival-order buffer, importance weights,
    optimiser with norm clipping): every weight, Adam moment and loss scalar must come out bit-identical: no
    result in the path depends on the order in which workgroups happen to run."""
    from paper_2210_05064_amd.learner import Learner
    w = wl.scaled(wl.WORKLOADS[name], hidden=128, input_dim=36)
    ro = wl.make_rollout(w, seed=77, bias_scale=0.1)
    logp_old = torch.from_numpy(ro["logp_noise"] - 1.0).cuda()
    runs = []
    for _ in range(2):
        L = Learner(ro, compute=compute, max_is=1.0, arrival=wl.arrival_order(ro["env_off"], seed=78),
                    adam_total_steps=100, adam=dict(max_grad_norm=0.5), want_grad_norm=True)
        L.set_logp_old(logp_old)
        L.update()
        L.update()
        torch.cuda.synchronize()
        assert not L.lstm_timed_out()
        runs.append([host(t).copy() for t in L.weights + L.exp_avg + L.exp_avg_sq + [L.scalars, L.grad_norm, L.adv]])
    for a, b in zip(*runs):
        assert np.array_equal(a, b)
