"""CPU oracle: multi-layer LSTM actor-critic, one sequence piece at a time.

TEST INFRASTRUCTURE ONLY.  fp64 numpy, no packing, no batching over pieces;
matrix-vector products are the only library step.  Nothing in the product path
may import this file; it shares no code with the HIP kernels.

What it follows: the policy of the paper's section 4 ("Architecture") and
section 3: the per-step input vector (visual embedding joined with the state
vector) goes through a 2-layer LSTM, and the LSTM output predicts the action
distribution and the value.  Back-propagation through time runs over the
sequences of section 2.2.  The LSTM itself is only cited, so this is the
standard cell:

    z = W_ih x_t + b_ih + W_hh h_{t-1} + b_hh        z = [z_i; z_f; z_g; z_o]
    i = sigm(z_i)  f = sigm(z_f)  g = tanh(z_g)  o = sigm(z_o)
    c_t = f * c_{t-1} + i * g          h_t = o * tanh(c_t)

Readings taken where the paper is silent: gate order i, f, g, o with two bias
vectors; layer l+1 reads h_t of layer l; no dropout, projection, peepholes or
normalisation; the heads are one linear map each from the top layer's h_t
(u = W_a h + b_a, v = w_v . h + b_v); a piece starts from the state handed in
(zeros when none is given).
"""
import numpy as np


def _sigm(x):
    return 1.0 / (1.0 + np.exp(-x))


def _f64(a):
    return np.asarray(a, np.float64)


def weights_f64(weights):
    """Deep copy of a weight dict with every array in fp64."""
    return {
        "layers": [{k: _f64(v) for k, v in layer.items()} for layer in weights["layers"]],
        "W_a": _f64(weights["W_a"]), "b_a": _f64(weights["b_a"]),
        "w_v": _f64(weights["w_v"]), "b_v": _f64(weights["b_v"]),
        "log_std": _f64(weights["log_std"]),
    }


def piece_forward(x, weights, h0=None, c0=None):
    """Forward over ONE piece.  x: [len, D]; h0, c0: [nl, H] or None.

    Returns (u [len, A], v [len], saved) where saved keeps what the backward
    pass needs: per layer the inputs, gates, cell and hidden states.
    """
    x = _f64(x)
    n_steps = x.shape[0]
    layers = weights["layers"]
    saved = []
    inp = x
    for l, lw in enumerate(layers):
        H = lw["W_hh"].shape[1]
        h_prev = np.zeros(H) if h0 is None else _f64(h0[l]).copy()
        c_prev = np.zeros(H) if c0 is None else _f64(c0[l]).copy()
        rec = {"x": inp, "h_in": h_prev.copy(), "c_in": c_prev.copy(),
               "i": np.zeros((n_steps, H)), "f": np.zeros((n_steps, H)),
               "g": np.zeros((n_steps, H)), "o": np.zeros((n_steps, H)),
               "c": np.zeros((n_steps, H)), "h": np.zeros((n_steps, H))}
        for t in range(n_steps):
            z = lw["W_ih"] @ inp[t] + lw["b_ih"] + lw["W_hh"] @ h_prev + lw["b_hh"]
            i = _sigm(z[0:H])
            f = _sigm(z[H:2 * H])
            g = np.tanh(z[2 * H:3 * H])
            o = _sigm(z[3 * H:4 * H])
            c = f * c_prev + i * g
            h = o * np.tanh(c)
            rec["i"][t], rec["f"][t], rec["g"][t], rec["o"][t] = i, f, g, o
            rec["c"][t], rec["h"][t] = c, h
            h_prev, c_prev = h, c
        saved.append(rec)
        inp = rec["h"]
    top = saved[-1]["h"]
    u = top @ weights["W_a"].T + weights["b_a"]
    v = top @ weights["w_v"] + weights["b_v"][0]
    return u, v, saved


def zero_grads(weights):
    g = {"layers": [{k: np.zeros_like(_f64(v)) for k, v in layer.items()} for layer in weights["layers"]]}
    for k in ("W_a", "b_a", "w_v", "b_v"):
        g[k] = np.zeros_like(_f64(weights[k]))
    return g


def piece_backward(d_u, d_v, weights, saved, grads):
    """Back-propagation through time over ONE piece.

    d_u [len, A], d_v [len]: gradient of the loss w.r.t. the heads' outputs.
    Adds this piece's weight gradients into `grads`; returns d_x [len, D].
    """
    d_u, d_v = _f64(d_u), _f64(d_v)
    layers = weights["layers"]
    n_steps = d_u.shape[0]
    top = saved[-1]["h"]
    # heads: u = W_a h + b_a, v = w_v . h + b_v
    for t in range(n_steps):
        grads["W_a"] += np.outer(d_u[t], top[t])
        grads["b_a"] += d_u[t]
        grads["w_v"] += d_v[t] * top[t]
        grads["b_v"] += d_v[t]
    d_above = d_u @ weights["W_a"] + np.outer(d_v, weights["w_v"])      # dL/dh_t of the top layer

    for l in range(len(layers) - 1, -1, -1):
        lw, rec, gl = layers[l], saved[l], grads["layers"][l]
        H = lw["W_hh"].shape[1]
        d_in = np.zeros_like(rec["x"])
        dh_rec = np.zeros(H)
        dc_rec = np.zeros(H)
        for t in range(n_steps - 1, -1, -1):
            i, f, g, o, c = rec["i"][t], rec["f"][t], rec["g"][t], rec["o"][t], rec["c"][t]
            c_prev = rec["c"][t - 1] if t > 0 else rec["c_in"]
            h_prev = rec["h"][t - 1] if t > 0 else rec["h_in"]
            tanh_c = np.tanh(c)
            dh = d_above[t] + dh_rec
            dc = dc_rec + dh * o * (1.0 - tanh_c * tanh_c)
            dz = np.concatenate([
                dc * g * i * (1.0 - i),            # input gate
                dc * c_prev * f * (1.0 - f),       # forget gate
                dc * i * (1.0 - g * g),            # cell candidate
                dh * tanh_c * o * (1.0 - o),       # output gate
            ])
            dc_rec = dc * f
            dh_rec = lw["W_hh"].T @ dz
            d_in[t] = lw["W_ih"].T @ dz
            gl["W_ih"] += np.outer(dz, rec["x"][t])
            gl["W_hh"] += np.outer(dz, h_prev)
            gl["b_ih"] += dz
            gl["b_hh"] += dz
        d_above = d_in
    return d_above


def minibatch_forward(x_steps, pieces_first, pieces_len, weights, h0=None, c0=None):
    """Runs every piece separately.  x_steps is the FLAT per-step input [S, D];
    piece j covers flat steps pieces_first[j] .. +pieces_len[j]-1.
    h0, c0: [nl, n_seq, H] or None.  Returns per-piece lists (u, v, saved)."""
    out = []
    for j, (first, n) in enumerate(zip(pieces_first, pieces_len)):
        first, n = int(first), int(n)
        hj = None if h0 is None else np.asarray(h0)[:, j, :]
        cj = None if c0 is None else np.asarray(c0)[:, j, :]
        out.append(piece_forward(np.asarray(x_steps)[first:first + n], weights, hj, cj))
    return out


def to_packed(per_piece, t_off):
    """Place per-piece rows [len_j, ...] at packed row t_off[t] + j."""
    M = int(t_off[-1])
    sample = np.asarray(per_piece[0])
    packed = np.zeros((M,) + sample.shape[1:], sample.dtype)
    for j, rows in enumerate(per_piece):
        for t in range(len(rows)):
            packed[int(t_off[t]) + j] = rows[t]
    return packed


def from_packed(packed, t_off, pieces_len):
    """Inverse of to_packed: list of [len_j, ...] arrays."""
    packed = np.asarray(packed)
    return [np.stack([packed[int(t_off[t]) + j] for t in range(int(n))]) for j, n in enumerate(pieces_len)]
