"""Pins for the LSTM + heads oracle: a library LSTM fed padded-then-packed
copies (forward and autograd backward), finite differences, order invariance,
state carry-over, degenerate closed forms.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import lstm
from paper_2210_05064_amd import workloads as wl


def small(seed, n_layers=2, H=5, D=3, A=4, bias_scale=0.3):
    w = wl.scaled(wl.WORKLOADS["tiny"], n_layers=n_layers, hidden=H, input_dim=D, act_dim=A)
    rng = np.random.default_rng(seed)
    weights = wl.make_weights(w, rng, bias_scale=bias_scale)
    return w, rng, lstm.weights_f64(weights)


def torch_lstm(weights, D, H, nl):
    net = torch.nn.LSTM(D, H, nl).double()
    with torch.no_grad():
        for l, lw in enumerate(weights["layers"]):
            getattr(net, f"weight_ih_l{l}").copy_(torch.from_numpy(lw["W_ih"]))
            getattr(net, f"weight_hh_l{l}").copy_(torch.from_numpy(lw["W_hh"]))
            getattr(net, f"bias_ih_l{l}").copy_(torch.from_numpy(lw["b_ih"]))
            getattr(net, f"bias_hh_l{l}").copy_(torch.from_numpy(lw["b_hh"]))
    return net


@pytest.mark.parametrize("seed", [0, 1])
def test_against_library_lstm_padded_then_packed(seed):
    w, rng, weights = small(seed)
    D, H, nl, A = w.input_dim, w.hidden, w.n_layers, w.act_dim
    lens = [7, 4, 4, 1]
    xs = [rng.standard_normal((n, D)) for n in lens]
    h0 = 0.5 * rng.standard_normal((nl, len(lens), H))
    c0 = 0.5 * rng.standard_normal((nl, len(lens), H))
    du = [rng.standard_normal((n, A)) for n in lens]
    dv = [rng.standard_normal(n) for n in lens]

    grads = lstm.zero_grads(weights)
    outs, dxs = [], []
    for j, x in enumerate(xs):
        u, v, saved = lstm.piece_forward(x, weights, h0[:, j], c0[:, j])
        outs.append((u, v))
        dxs.append(lstm.piece_backward(du[j], dv[j], weights, saved, grads))

    net = torch_lstm(weights, D, H, nl)
    Wa = torch.tensor(weights["W_a"], requires_grad=True)
    ba = torch.tensor(weights["b_a"], requires_grad=True)
    wv = torch.tensor(weights["w_v"], requires_grad=True)
    bv = torch.tensor(weights["b_v"], requires_grad=True)
    xt = [torch.tensor(x, requires_grad=True) for x in xs]
    packed = torch.nn.utils.rnn.pack_sequence(xt, enforce_sorted=True)
    y, _ = net(packed, (torch.tensor(h0), torch.tensor(c0)))
    y, _ = torch.nn.utils.rnn.pad_packed_sequence(y)          # [T, n, H]
    loss = 0.0
    for j, n in enumerate(lens):
        hj = y[:n, j]
        u_t = hj @ Wa.T + ba
        v_t = hj @ wv + bv
        np.testing.assert_allclose(outs[j][0], u_t.detach().numpy(), atol=1e-12)
        np.testing.assert_allclose(outs[j][1], v_t.detach().numpy(), atol=1e-12)
        loss = loss + (u_t * torch.tensor(du[j])).sum() + (v_t * torch.tensor(dv[j])).sum()
    loss.backward()
    for l in range(nl):
        for ours, theirs in (("W_ih", "weight_ih"), ("W_hh", "weight_hh"), ("b_ih", "bias_ih"), ("b_hh", "bias_hh")):
            np.testing.assert_allclose(grads["layers"][l][ours], getattr(net, f"{theirs}_l{l}").grad.numpy(),
                                       atol=1e-11)
    np.testing.assert_allclose(grads["W_a"], Wa.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(grads["b_a"], ba.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(grads["w_v"], wv.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(grads["b_v"], bv.grad.numpy(), atol=1e-11)
    for j in range(len(lens)):
        np.testing.assert_allclose(dxs[j], xt[j].grad.numpy(), atol=1e-11)


def scalar_objective(weights, xs, h0, c0, du, dv):
    tot = 0.0
    for j, x in enumerate(xs):
        u, v, _ = lstm.piece_forward(x, weights, h0[:, j], c0[:, j])
        tot += np.sum(u * du[j]) + np.sum(v * dv[j])
    return tot


def test_finite_differences_every_tensor():
    w, rng, weights = small(5)
    D, H, nl, A = w.input_dim, w.hidden, w.n_layers, w.act_dim
    lens = [6, 3]
    xs = [rng.standard_normal((n, D)) for n in lens]
    h0 = 0.3 * rng.standard_normal((nl, 2, H))
    c0 = 0.3 * rng.standard_normal((nl, 2, H))
    du = [rng.standard_normal((n, A)) for n in lens]
    dv = [rng.standard_normal(n) for n in lens]
    grads = lstm.zero_grads(weights)
    for j, x in enumerate(xs):
        _, _, saved = lstm.piece_forward(x, weights, h0[:, j], c0[:, j])
        lstm.piece_backward(du[j], dv[j], weights, saved, grads)
    eps = 1e-6
    tensors = [(weights[k], grads[k]) for k in ("W_a", "b_a", "w_v", "b_v")]
    for l in range(nl):
        tensors += [(weights["layers"][l][k], grads["layers"][l][k]) for k in ("W_ih", "W_hh", "b_ih", "b_hh")]
    for arr, g in tensors:
        flat, gflat = arr.reshape(-1), g.reshape(-1)
        for idx in rng.choice(flat.size, size=min(6, flat.size), replace=False):
            keep = flat[idx]
            flat[idx] = keep + eps
            up = scalar_objective(weights, xs, h0, c0, du, dv)
            flat[idx] = keep - eps
            dn = scalar_objective(weights, xs, h0, c0, du, dv)
            flat[idx] = keep
            fd = (up - dn) / (2 * eps)
            assert abs(fd - gflat[idx]) <= 1e-6 * max(1.0, abs(fd)), (fd, gflat[idx])


def test_piece_order_does_not_matter():
    w, rng, weights = small(7)
    lens = [5, 2, 9, 1]
    xs = [rng.standard_normal((n, w.input_dim)) for n in lens]
    du = [rng.standard_normal((n, w.act_dim)) for n in lens]
    dv = [rng.standard_normal(n) for n in lens]

    def run(order):
        grads = lstm.zero_grads(weights)
        outs = {}
        for j in order:
            u, v, saved = lstm.piece_forward(xs[j], weights)
            lstm.piece_backward(du[j], dv[j], weights, saved, grads)
            outs[j] = u
        return outs, grads
    o1, g1 = run([0, 1, 2, 3])
    o2, g2 = run([2, 0, 3, 1])
    for j in range(4):
        assert np.array_equal(o1[j], o2[j])
    np.testing.assert_allclose(g1["layers"][0]["W_hh"], g2["layers"][0]["W_hh"], atol=1e-13)
    np.testing.assert_allclose(g1["layers"][1]["W_ih"], g2["layers"][1]["W_ih"], atol=1e-13)


def test_split_piece_with_carried_state():
    """Cutting a piece in two and starting the tail from the head's final
    state reproduces the unsplit forward."""
    w, rng, weights = small(8)
    x = rng.standard_normal((9, w.input_dim))
    u, v, saved = lstm.piece_forward(x, weights)
    cut = 4
    hT = np.stack([saved[l]["h"][cut - 1] for l in range(w.n_layers)])
    cT = np.stack([saved[l]["c"][cut - 1] for l in range(w.n_layers)])
    u2, v2, _ = lstm.piece_forward(x[cut:], weights, hT, cT)
    np.testing.assert_allclose(u2, u[cut:], atol=1e-14)
    np.testing.assert_allclose(v2, v[cut:], atol=1e-14)


def test_zero_recurrent_weights_is_a_gated_mlp():
    w, rng, weights = small(9, n_layers=1)
    weights["layers"][0]["W_hh"][:] = 0
    H = w.hidden
    x = rng.standard_normal((4, w.input_dim))
    _, _, saved = lstm.piece_forward(x, weights)
    lw = weights["layers"][0]
    sg = lambda a: 1 / (1 + np.exp(-a))
    c_prev = np.zeros(H)
    for t in range(4):
        z = lw["W_ih"] @ x[t] + lw["b_ih"] + lw["b_hh"]
        c_prev = sg(z[H:2 * H]) * c_prev + sg(z[:H]) * np.tanh(z[2 * H:3 * H])
        np.testing.assert_allclose(saved[0]["h"][t], sg(z[3 * H:]) * np.tanh(c_prev), atol=1e-15)


def test_saturated_gates_hold_the_cell():
    """Forget bias -> +inf and input bias -> -inf keep c_t = c_0."""
    w, rng, weights = small(10, n_layers=1)
    H = w.hidden
    weights["layers"][0]["b_ih"][:H] = -60.0
    weights["layers"][0]["b_ih"][H:2 * H] = 60.0
    c0 = rng.standard_normal((1, H))
    _, _, saved = lstm.piece_forward(rng.standard_normal((5, w.input_dim)), weights, np.zeros((1, H)), c0)
    np.testing.assert_allclose(saved[0]["c"][-1], c0[0], atol=1e-12)


def test_packed_placement_round_trip():
    t_off = np.array([0, 3, 5, 6])
    lens = [3, 2, 1]
    pieces = [np.arange(n, dtype=np.float64) + 10 * j for j, n in enumerate(lens)]
    packed = lstm.to_packed(pieces, t_off)
    assert packed.tolist() == [0, 10, 20, 1, 11, 2]
    back = lstm.from_packed(packed, t_off, lens)
    assert all(np.array_equal(a, b) for a, b in zip(back, pieces))
