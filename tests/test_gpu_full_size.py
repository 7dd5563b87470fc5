"""Parity at the workloads' FULL sizes, in the launch configuration bench.py
times (same Learner, same kernels): integer outputs and copies bit-exact on the
whole minibatch, LSTM outputs and gradients on a sample of pieces the oracle
can afford (a piece's outputs depend on that piece alone, and with the loss
gradient confined to the sampled pieces the weight gradients are exactly the
sum over those pieces).  The sample holds the minibatch's LONGEST piece (hundreds
of dependent timesteps at full width, the last of them at batch size 1), a piece
of middle rank and the shortest ones."""
import numpy as np
import pytest
import torch

from oracle import gae as ogae, lstm as olstm, pack as opack
from paper_2210_05064_amd import workloads as wl
from tests.gpu_util import GRAD_NAMES, grads_to_list, host
from tests.util import assert_close, closer

pytestmark = pytest.mark.gpu


def sample_pieces(meta, max_steps):
    """All pieces if the minibatch has at most max_steps rows; else the longest piece (rank 0), pieces at the
    middle, quarter and eighth ranks of the longest-first order, and the shortest pieces (the end of that order)
    while the total stays within max_steps."""
    n = meta["n_seq"]
    if meta["M"] <= max_steps:
        return list(range(n))
    chosen = []
    for j in (0, n // 2, n // 4, (3 * n) // 4, n // 8):
        if j not in chosen:
            chosen.append(j)
    total = sum(int(meta["seq_len"][j]) for j in chosen)
    for j in range(n - 1, -1, -1):
        ln = int(meta["seq_len"][j])
        if j in chosen:
            continue
        if total + ln > max_steps:
            break
        chosen.append(j)
        total += ln
    return chosen


@pytest.mark.parametrize("name,max_steps", [("nav", 1024), ("manip", 1024), ("large", 2048), ("max", 2000)])
def test_full_size_minibatch(ver, name, max_steps):
    from paper_2210_05064_amd.learner import Learner
    w = wl.WORKLOADS[name]
    ro = wl.make_rollout(w, seed=77, bias_scale=0.05)
    L = Learner(ro, want_dx=True)
    rng = np.random.default_rng(5)
    L.logp_old.copy_(torch.from_numpy(rng.standard_normal(ro["S"]).astype(np.float32)).cuda())
    e, b = w.epochs - 1, w.minibatches - 1
    L.gae()
    L.pack(e, b)
    L.forward()
    torch.cuda.synchronize()
    assert not L.lstm_timed_out()

    # advantages, packing and gathers: the whole thing, exactly
    adv, ret = ogae.gae(ro["rewards"], ro["values"], ro["dones"], ro["last_values"], ro["env_off"], w.gamma, w.lam)
    assert_close(host(L.adv), adv, 1e-5, "adv")
    meta = opack.pack_minibatch(ro["dones"], ro["env_off"], ro["seq_key"][e], w.minibatches, b, ro["env_started_episode"])
    assert host(L.info).tolist()[:3] == [meta["n_seq"], meta["T_max"], meta["K"]]
    g = meta["gather_idx"]
    assert np.array_equal(host(L.gather_idx), g)
    assert np.array_equal(host(L.batch_sizes)[:meta["T_max"]], meta["batch_sizes"])
    x_ref = torch.from_numpy(ro["obs"][g])
    assert torch.equal(L.x_packed.cpu(), x_ref.to(torch.bfloat16) if L.x_bf16 else x_ref)
    assert np.array_equal(host(L.act_packed), ro["actions"][g])
    n = meta["n_seq"]
    h0 = opack.initial_states(ro["rnn_h"], meta["seq_first"], meta["seq_is_ep_start"])
    c0 = opack.initial_states(ro["rnn_c"], meta["seq_first"], meta["seq_is_ep_start"])
    assert np.array_equal(host(L.h0)[:, :n], h0) and np.array_equal(host(L.c0)[:, :n], c0)

    # LSTM: sampled pieces
    chosen = sample_pieces(meta, max_steps)
    assert len(chosen) >= 3 and 0 in chosen and int(meta["seq_len"][0]) == meta["T_max"]
    W = olstm.weights_f64(ro["weights"])
    rows = {j: [int(meta["t_off"][t]) + j for t in range(int(meta["seq_len"][j]))] for j in chosen}
    d_u = np.zeros((L.M, w.act_dim), np.float32)
    d_v = np.zeros(L.M, np.float32)
    for j in chosen:
        d_u[rows[j]] = rng.standard_normal((len(rows[j]), w.act_dim)) / 64
        d_v[rows[j]] = rng.standard_normal(len(rows[j])) / 64
    L.d_head.copy_(torch.from_numpy(d_u).cuda())
    L.d_value.copy_(torch.from_numpy(d_v).cuda())
    L.backward()
    torch.cuda.synchronize()
    assert not L.lstm_timed_out()

    close = closer(L.compute)
    grads = olstm.zero_grads(W)
    u_gpu, v_gpu, dx_gpu = host(L.head_out), host(L.value), host(L.d_x)
    u_ref, v_ref, dx_ref, idx = [], [], [], []
    for j in chosen:
        f0, ln = int(meta["seq_first"][j]), int(meta["seq_len"][j])
        u, v, saved = olstm.piece_forward(ro["obs"][f0:f0 + ln], W, h0[:, j], c0[:, j])
        dx = olstm.piece_backward(d_u[rows[j]], d_v[rows[j]], W, saved, grads)
        u_ref.append(u); v_ref.append(v); dx_ref.append(dx); idx += rows[j]
    close(u_gpu[idx], np.concatenate(u_ref), "head_out (sampled pieces)")
    close(v_gpu[idx], np.concatenate(v_ref), "value (sampled pieces)")
    close(dx_gpu[idx], np.concatenate(dx_ref), "d_x (sampled pieces)")
    others = np.setdiff1d(np.arange(L.M), np.array(idx))
    assert np.all(dx_gpu[others] == 0), "no gradient may reach pieces outside the sample"
    names = [f"layer{l}.{nme}" for l in range(w.n_layers) for nme in GRAD_NAMES] + ["W_a", "b_a", "w_v", "b_v"]
    for nme, gg, r in zip(names, L.grads, grads_to_list(grads)):
        close(host(gg), r, nme)


@pytest.mark.parametrize("name", ["large", "max"])
def test_full_size_two_layer_launch_matches_layer_by_layer(ver, name):
    """The whole minibatch at full width through both launch modes (both time loops in one launch, as bench.py
    times it, and one launch per layer): they differ in the order of fp32 additions in the projection between the
    layers, after which a last-bit difference can flip the bf16 rounding of an operand (2^-9 relative)."""
    from paper_2210_05064_amd.learner import Learner
    from tests.util import rel_err
    w = wl.WORKLOADS[name]
    ro = wl.make_rollout(w, seed=78, bias_scale=0.05)
    rng = np.random.default_rng(6)
    M = ro["S"] // w.minibatches
    d_u = torch.from_numpy((rng.standard_normal((M, w.act_dim)) / M).astype(np.float32)).cuda()
    d_v = torch.from_numpy((rng.standard_normal(M) / M).astype(np.float32)).cuda()
    res = []
    for layer_by_layer in (False, True):
        L = Learner(ro, want_dx=True, layer_by_layer=layer_by_layer)
        L.gae()
        L.pack(0, 1)
        L.forward()
        L.d_head.copy_(d_u)
        L.d_value.copy_(d_v)
        L.backward()
        torch.cuda.synchronize()
        assert not L.lstm_timed_out()
        res.append([host(t) for t in [L.head_out, L.value, L.d_x] + L.grads])
        del L
    names = ["head_out", "value", "d_x"] + [f"grad[{i}]" for i in range(len(res[0]) - 3)]
    for nme, a, b in zip(names, *res):
        assert np.all(np.isfinite(a)) and rel_err(a, b) < 2e-2, (nme, rel_err(a, b))


@pytest.mark.parametrize("name", ["large", "max"])
def test_full_size_optimizer_step_and_weights(ver, name):
    """The steps that surround the minibatch loop at full size, in the configuration bench.py times: the Adam step
    over every weight tensor of the workload's network (the oracle is elementwise numpy: all 17 M parameters of
    `max` are compared, not a sample), the importance weights of the whole buffer, and the bucketing of the
    arrival-order buffer."""
    from oracle import adam as oadam, ingest as oing, is_weight as ois
    from paper_2210_05064_amd.learner import Learner
    w = wl.WORKLOADS[name]
    ro = wl.make_rollout(w, seed=3, with_states=False)
    arr = wl.arrival_order(ro["env_off"], seed=4)
    L = Learner(ro, adam_total_steps=1000, max_is=1.0, arrival=arr, want_grad_norm=True)
    # bucketing and importance weights
    L.ingest()
    L.importance_weights()
    torch.cuda.synchronize()
    r_off, r_order, _ = oing.ingest(arr[0], ro["N"], arr[1])
    assert np.array_equal(host(L.env_off), r_off) and np.array_equal(host(L.order), r_order)
    assert host(L.ingest_info).tolist() == [0, 0, 0, 0]
    assert np.array_equal(host(L.obs), ro["obs"]) and np.array_equal(host(L.dones), ro["dones"])
    assert np.array_equal(host(L.is_w), ois.is_weights(ro["env_off"], 1.0).astype(np.float32))
    # one optimiser step on seeded gradients
    rng = np.random.default_rng(5)
    grads = [(rng.standard_normal(tuple(t.shape)) * 10.0 ** rng.integers(-3, 1)).astype(np.float32) for t in L.opt_params]
    for g_dev, g in zip(L.opt_grads, grads):
        g_dev.copy_(torch.from_numpy(g).cuda())
    before = [host(t).astype(np.float64) for t in L.opt_params]
    L.opt_steps = 37
    L.optimizer_step()
    torch.cuda.synchronize()
    f32 = lambda x: float(np.float32(x))
    lr = oadam.cosine_lr(37, 1000, f32(2.5e-4), 0.0)
    new_p, new_m, new_v, norm = oadam.adam_step(before, grads, [np.zeros_like(b) for b in before],
                                                [np.zeros_like(b) for b in before], 38, lr, f32(0.9), f32(0.999), f32(1e-8))
    assert float(L.grad_norm.item()) == pytest.approx(norm, rel=1e-5)
    n_params = 0
    for i, t in enumerate(L.opt_params):
        # the step is ~lr while the weights are ~1e-2: compare the moments exactly and the change of the weights
        # to the resolution fp32 leaves of it
        assert_close(host(L.exp_avg[i]), new_m[i], 1e-5, f"m[{i}]")
        assert_close(host(L.exp_avg_sq[i]), new_v[i], 1e-5, f"v[{i}]")
        got, want = host(t).astype(np.float64) - before[i], new_p[i] - before[i]
        assert np.max(np.abs(got - want)) <= 2.0 ** -24 * max(1e-30, float(np.max(np.abs(before[i])))) + 1e-5 * np.max(np.abs(want))
        n_params += t.numel()
    assert n_params == sum(b.size for b in before) and n_params > (10 ** 7 if name == "max" else 10 ** 6)
