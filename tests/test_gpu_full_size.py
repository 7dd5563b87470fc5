"""Parity at the workloads' FULL sizes, in the launch configuration bench.py
times (same Learner, same kernels): integer outputs and copies bit-exact on the
whole minibatch, LSTM outputs and gradients on a sample of pieces the oracle
can afford (a piece's outputs depend on that piece alone, and with the loss
gradient confined to the sampled pieces the weight gradients are exactly the
sum over those pieces)."""
import numpy as np
import pytest
import torch

from oracle import gae as ogae, lstm as olstm, pack as opack
from paper_2210_05064_amd import workloads as wl
from tests.gpu_util import GRAD_NAMES, grads_to_list, host
from tests.util import assert_close, assert_close_bf16

pytestmark = pytest.mark.gpu


def sample_pieces(meta, max_steps):
    """Shortest pieces first (they sit at the end of the longest-first order), a few mid-sized ones too."""
    order = list(range(meta["n_seq"] - 1, -1, -1))
    chosen, total = [], 0
    for j in order:
        n = int(meta["seq_len"][j])
        if total + n > max_steps:
            break
        chosen.append(j)
        total += n
    return chosen


@pytest.mark.parametrize("name,max_steps", [("nav", 60), ("manip", 60), ("large", 60), ("max", 24)])
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
    assert len(chosen) >= 2
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

    close = (lambda a, r, nme: assert_close(a, r, 1e-4, nme)) if L.compute == 0 else assert_close_bf16
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
