"""ver_lstm_fwd / ver_lstm_bwd against the CPU oracle (unpacked, per piece,
fp64).  fp32 path: every element within 1e-4 of max(|ref|, rms(ref)).
bf16-operand path: every element within 2e-2 in the same metric, except the
tensors that come out of back-propagation through time, which have a bar of
their own (tests/util.py: assert_close_bf16_bptt)."""
import numpy as np
import pytest

from oracle import lstm as olstm, pack as opack
from paper_2210_05064_amd import workloads as wl
from tests.gpu_util import LstmRun, grads_to_list, GRAD_NAMES
from tests.util import closer, rel_err

pytestmark = pytest.mark.gpu


def oracle_run(ro, w, meta, h0, c0, d_u, d_v):
    W = olstm.weights_f64(ro["weights"])
    fwd = olstm.minibatch_forward(ro["obs"], meta["seq_first"], meta["seq_len"], W, h0, c0)
    u = olstm.to_packed([f[0] for f in fwd], meta["t_off"])
    v = olstm.to_packed([f[1] for f in fwd], meta["t_off"])
    grads = olstm.zero_grads(W)
    du_p = olstm.from_packed(d_u, meta["t_off"], meta["seq_len"])
    dv_p = olstm.from_packed(d_v, meta["t_off"], meta["seq_len"])
    dx = [olstm.piece_backward(du_p[j], dv_p[j], W, fwd[j][2], grads) for j in range(meta["n_seq"])]
    return u, v, grads, olstm.to_packed(dx, meta["t_off"])


def case(ver, w, seed, b=0, compute=0, x_bf16=False, states=True, bias_scale=0.2, layer_by_layer=False):
    ro = wl.make_rollout(w, seed=seed, bias_scale=bias_scale)
    B = w.minibatches
    meta = opack.pack_minibatch(ro["dones"], ro["env_off"], ro["seq_key"][0], B, b, ro["env_started_episode"])
    h0 = c0 = None
    if states:
        h0 = opack.initial_states(ro["rnn_h"], meta["seq_first"], meta["seq_is_ep_start"])
        c0 = opack.initial_states(ro["rnn_c"], meta["seq_first"], meta["seq_is_ep_start"])
    rng = np.random.default_rng(seed + 1)
    M = meta["M"]
    d_u = (rng.standard_normal((M, w.act_dim)) / M).astype(np.float32)
    d_v = (rng.standard_normal(M) / M).astype(np.float32)
    x_packed = opack.gather_rows(ro["obs"], meta["gather_idx"])
    run = LstmRun(ver, w, ro["weights"], x_packed, meta, h0, c0, compute, x_bf16, layer_by_layer)
    u, v = run.forward()
    grads, d_x = run.backward(d_u, d_v)
    r_u, r_v, r_grads, r_dx = oracle_run(ro, w, meta, h0, c0, d_u, d_v)
    close = closer(compute)
    close(u, r_u, "head_out")
    close(v, r_v, "value")
    close(d_x, r_dx, "d_x")
    names = [f"layer{l}.{n}" for l in range(w.n_layers) for n in GRAD_NAMES] + ["W_a", "b_a", "w_v", "b_v"]
    for name, g, r in zip(names, grads, grads_to_list(r_grads)):
        close(g, r, name)
    return run, meta


SMALL = dict(budget=640, n_envs=12, hidden=128, input_dim=36, p_done=0.02, minibatches=2)


@pytest.mark.parametrize("compute", [0, 1])
@pytest.mark.parametrize("b", [0, 1])
def test_two_layers_ragged(ver, compute, b):
    """Several MFMA tiles in every dimension, ragged tail of single pieces,
    initial states, both minibatches (the second opens with a split piece)."""
    case(ver, wl.scaled(wl.WORKLOADS["manip"], **SMALL), seed=21, b=b, compute=compute)


@pytest.mark.parametrize("compute", [0, 1])
def test_two_layers_one_launch_per_layer(ver, compute):
    """Two-layer networks normally run both time loops in one launch; the layer-by-layer path (every other
    depth) is checked against the oracle on the same case through the library's diagnostic switch."""
    case(ver, wl.scaled(wl.WORKLOADS["manip"], **SMALL), seed=21, b=1, compute=compute, layer_by_layer=True)


@pytest.mark.parametrize("compute", [0, 1])
def test_two_layer_launch_matches_layer_by_layer(ver, compute):
    """Same inputs through both paths: they differ only in the order of fp32 additions in the projection
    between the layers."""
    w = wl.scaled(wl.WORKLOADS["manip"], budget=1500, n_envs=70, hidden=128, input_dim=36, p_done=0.03, minibatches=1)
    ro = wl.make_rollout(w, seed=31, bias_scale=0.2)
    meta = opack.pack_minibatch(ro["dones"], ro["env_off"], ro["seq_key"][0], 1, 0, ro["env_started_episode"])
    h0 = opack.initial_states(ro["rnn_h"], meta["seq_first"], meta["seq_is_ep_start"])
    c0 = opack.initial_states(ro["rnn_c"], meta["seq_first"], meta["seq_is_ep_start"])
    rng = np.random.default_rng(2)
    d_u = (rng.standard_normal((meta["M"], w.act_dim)) / meta["M"]).astype(np.float32)
    d_v = (rng.standard_normal(meta["M"]) / meta["M"]).astype(np.float32)
    res = []
    for layer_by_layer in (False, True):
        run = LstmRun(ver, w, ro["weights"], opack.gather_rows(ro["obs"], meta["gather_idx"]), meta, h0, c0, compute,
                      layer_by_layer=layer_by_layer)
        u, v = run.forward()
        grads, dx = run.backward(d_u, d_v)
        res.append([u, v, dx] + grads)
    for a, b in zip(*res):
        # bf16 operands: a last-bit difference in fp32 can flip the rounding of an operand (2^-9 relative)
        assert rel_err(a, b) < (1e-5 if compute == 0 else 1e-2)


@pytest.mark.parametrize("compute", [0, 1])
def test_tiny_workload(ver, compute):
    case(ver, wl.WORKLOADS["tiny"], seed=3, compute=compute)


def test_categorical_no_initial_state_bf16_input(ver):
    case(ver, wl.scaled(wl.WORKLOADS["nav"], budget=512, n_envs=8, hidden=64, input_dim=20, p_done=0.05),
         seed=5, compute=1, x_bf16=True, states=False)


@pytest.mark.parametrize("compute", [0, 1])
def test_many_short_pieces(ver, compute):
    """More pieces than one MFMA tile holds (n_seq > 16) and T_max small."""
    case(ver, wl.scaled(wl.WORKLOADS["nav"], budget=600, n_envs=40, hidden=64, input_dim=12, p_done=0.2,
                        minibatches=1, speed_sigma=0.3), seed=6, compute=compute)


def test_single_long_piece(ver):
    """One environment owns the minibatch: batch size 1 at every timestep."""
    case(ver, wl.scaled(wl.WORKLOADS["nav"], budget=300, n_envs=1, hidden=64, input_dim=8, p_done=0.0,
                        minibatches=1), seed=7)


@pytest.mark.parametrize("compute", [0, 1])
def test_two_pieces_leave_a_group_empty(ver, compute):
    """Two-layer launch with fewer pieces than groups: the third group has no piece and no timestep."""
    case(ver, wl.scaled(wl.WORKLOADS["nav"], budget=200, n_envs=2, hidden=64, input_dim=8, p_done=0.0,
                        minibatches=1, speed_sigma=1.0), seed=11, compute=compute)


@pytest.mark.parametrize("n_envs", [3000, 5000])
def test_thousands_of_pieces(ver, n_envs):
    """Two-layer launch over thousands of pieces of 2 timesteps: the plan's prefix sums run over several blocks of
    pieces (held in LDS up to 4096 pieces, in global memory beyond), a group holds more than 64 tiles of 16 pieces,
    a timestep of a group more rows than a GEMM tile."""
    _, meta = case(ver, wl.scaled(wl.WORKLOADS["nav"], budget=2 * n_envs, n_envs=n_envs, hidden=64, input_dim=8, p_done=0.0,
                                  minibatches=1, speed_sigma=0.0), seed=12, compute=1)
    assert meta["n_seq"] >= n_envs


def test_long_and_short_pieces(ver):
    """Two-layer launch with more than 1024 timesteps (the plan's row prefix runs over several blocks of
    timesteps) and pieces of very different lengths."""
    _, meta = case(ver, wl.scaled(wl.WORKLOADS["nav"], budget=3000, n_envs=6, hidden=64, input_dim=8, p_done=0.001,
                                  minibatches=1, speed_sigma=1.5), seed=13, compute=0)
    assert meta["T_max"] > 1024


def test_wide_hidden_not_a_multiple_of_128(ver):
    """hidden = 576 (bf16 operands; fp32 keeps its share of W_hh in registers only up to hidden = 512): more than 32
    tiles of 16 units (workgroups of 32 units) and a contraction that does not split into whole operand blocks four
    ways: the general (not width-specialised) forms of both time loops."""
    case(ver, wl.scaled(wl.WORKLOADS["manip"], budget=200, n_envs=5, hidden=576, input_dim=20, p_done=0.02,
                        minibatches=1), seed=17, compute=1)


@pytest.mark.parametrize("seed", range(12))
def test_two_layer_launch_random_packings(ver, seed):
    """The plan of the two-layer launch (which pieces a group runs, its chunks, the gathered rows of the workers'
    tiles) over packings of very different shape: 1 to 60 environments, 40 to 900 rows, few to many episode ends."""
    rng = np.random.default_rng(1000 + seed)
    n_envs = int(rng.integers(1, 61))
    budget = int(rng.integers(max(40, 2 * n_envs), 901))
    w = wl.scaled(wl.WORKLOADS["nav"], budget=budget, n_envs=n_envs, hidden=64, input_dim=8,
                  p_done=float(rng.choice([0.0, 0.01, 0.05, 0.3])), minibatches=1, speed_sigma=float(rng.choice([0.0, 0.5, 1.5])))
    case(ver, w, seed=50 + seed, compute=int(seed % 2))


def test_three_layers_wide_input(ver):
    case(ver, wl.scaled(wl.WORKLOADS["manip"], budget=256, n_envs=6, hidden=192, input_dim=260, n_layers=3,
                        p_done=0.03, minibatches=1), seed=8)


def test_packing_order_invariance_on_device(ver):
    """Another random order of the same sequences (B = 1): identical weight gradients up to rounding."""
    w = wl.scaled(wl.WORKLOADS["manip"], budget=400, n_envs=10, hidden=64, input_dim=16, p_done=0.03,
                  minibatches=1, epochs=2)
    ro = wl.make_rollout(w, seed=9, bias_scale=0.2)
    rng = np.random.default_rng(1)
    du_flat = (rng.standard_normal((ro["S"], w.act_dim)) / ro["S"]).astype(np.float32)
    dv_flat = (rng.standard_normal(ro["S"]) / ro["S"]).astype(np.float32)
    outs = []
    for e in range(2):
        meta = opack.pack_minibatch(ro["dones"], ro["env_off"], ro["seq_key"][e], 1, 0)
        g = meta["gather_idx"]
        run = LstmRun(ver, w, ro["weights"], ro["obs"][g], meta)
        u, v = run.forward()
        grads, _ = run.backward(du_flat[g], dv_flat[g])
        flat_u = np.zeros_like(u)
        flat_u[g] = u
        outs.append((flat_u, grads))
    assert rel_err(outs[0][0], outs[1][0]) < 1e-5
    for a, b in zip(outs[0][1], outs[1][1]):
        assert rel_err(a, b) < 1e-4


def test_bitwise_reproducible(ver):
    w = wl.scaled(wl.WORKLOADS["manip"], **SMALL)
    ro = wl.make_rollout(w, seed=4)
    meta = opack.pack_minibatch(ro["dones"], ro["env_off"], ro["seq_key"][0], 2, 0)
    rng = np.random.default_rng(0)
    d_u = rng.standard_normal((meta["M"], w.act_dim)).astype(np.float32)
    d_v = rng.standard_normal(meta["M"]).astype(np.float32)
    res = []
    for _ in range(2):
        run = LstmRun(ver, w, ro["weights"], ro["obs"][meta["gather_idx"]], meta, compute=1)
        u, v = run.forward()
        grads, dx = run.backward(d_u, d_v)
        res.append([u, v, dx] + grads)
    assert all(np.array_equal(a, b) for a, b in zip(*res))


def test_unsupported_shapes(ver):
    for kw in (dict(hidden=96), dict(hidden=1024), dict(input_dim=6), dict(n_layers=9)):
        c = dict(n_layers=1, input_dim=8, hidden=64, act_dim=4)
        c.update(kw)
        cfg = ver.lstm_cfg(c["n_layers"], c["input_dim"], c["hidden"], c["act_dim"], 0, 0)
        assert ver.ver_lstm_workspace_bytes(cfg, 16) == 0


@pytest.mark.parametrize("input_dim", [4, 60, 64, 68, 124, 128, 196])
def test_bf16_input_projection_any_width(ver, input_dim):
    """bf16 rows into the first layer: the projection walks the input width in tiles of 64, so widths just below,
    at and just above a multiple of 64 (and narrower than one tile), over three row tiles with a ragged last one."""
    case(ver, wl.scaled(wl.WORKLOADS["large"], budget=300, n_envs=5, hidden=64, input_dim=input_dim, p_done=0.02,
                        minibatches=1), seed=40 + input_dim, compute=1, x_bf16=True)


@pytest.mark.parametrize("input_dim,layer_by_layer", [(516, False), (1044, False), (544, False), (548, False), (1056, True),
                                                      (512, False), (640, True)])
def test_grouped_weight_gradients(ver, input_dim, layer_by_layer):
    """bf16 operands at a hidden size whose weight gradients leave in one grouped launch (4H a multiple of 1024),
    over input widths on both sides of its rules: a few columns beyond the last whole 128-column tile ride along
    with the whole tiles (4 or 20 columns beyond four whole tiles: two 16-row slices per tile; 20 or 32 beyond
    eight: one), more than 32 columns or no remainder take column tiles of their own."""
    case(ver, wl.scaled(wl.WORKLOADS["manip"], budget=420, n_envs=9, hidden=256, input_dim=input_dim, p_done=0.02,
                        minibatches=1), seed=41, compute=1, x_bf16=True, layer_by_layer=layer_by_layer)
