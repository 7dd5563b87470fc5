"""Helpers for the GPU parity tests: host arrays -> device tensors -> C-ABI calls."""
import numpy as np
import torch


def dev(a):
    """numpy array -> contiguous device tensor of the same dtype (uint32 travels as int32 bits)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def host(t):
    return t.detach().cpu().numpy()


def run_gae(ver, r, v, d, lv, off, gamma, lam):
    S, N = len(r), len(off) - 1
    adv = torch.full((max(S, 1),), float("nan"), device="cuda")
    ret = torch.full((max(S, 1),), float("nan"), device="cuda")
    ws = ver.workspace(ver.ver_gae_workspace_bytes(S))
    ws.fill_(-1)       # the library must not rely on workspace contents
    ver.ver_gae(dev(np.asarray(r, np.float32)), dev(np.asarray(v, np.float32)), dev(np.asarray(d, np.uint8)),
                dev(np.asarray(lv, np.float32)), dev(np.asarray(off, np.int32)), N, S, gamma, lam, adv, ret, ws)
    torch.cuda.synchronize()
    if S:
        assert ws[1].item() == 0, "device-side wait timed out"
    return host(adv)[:S], host(ret)[:S]


class PackOut:
    """Device buffers for one ver_pack_minibatch call, sized for the upper bound M."""

    def __init__(self, M, D=0, act_shape=(), act_dtype=torch.int32, nl=0, H=0, bf16=False):
        i32 = dict(dtype=torch.int32, device="cuda")
        self.M = M
        self.info = torch.full((4,), -7, **i32)
        self.seq_first = torch.full((M,), -7, **i32)
        self.seq_len = torch.full((M,), -7, **i32)
        self.seq_is_ep_start = torch.full((M,), 9, dtype=torch.uint8, device="cuda")
        self.batch_sizes = torch.full((M,), -7, **i32)
        self.t_off = torch.full((M + 1,), -7, **i32)
        self.gather_idx = torch.full((M,), -7, **i32)
        self.obs_packed = (torch.zeros((M, D), dtype=torch.bfloat16 if bf16 else torch.float32, device="cuda")
                           if D else None)
        self.actions_packed = torch.zeros((M,) + tuple(act_shape), dtype=act_dtype, device="cuda")
        self.logp_old_packed = torch.zeros(M, device="cuda")
        self.adv_packed = torch.zeros(M, device="cuda")
        self.ret_packed = torch.zeros(M, device="cuda")
        self.is_weight_packed = torch.zeros(M, device="cuda")
        self.h0 = torch.full((nl, M, H), float("nan"), device="cuda") if nl else None
        self.c0 = torch.full((nl, M, H), float("nan"), device="cuda") if nl else None

    def meta(self):
        n_seq, t_max, K, _ = host(self.info).tolist()
        return {
            "K": K, "n_seq": n_seq, "T_max": t_max, "M": self.M,
            "seq_first": host(self.seq_first)[:n_seq], "seq_len": host(self.seq_len)[:n_seq],
            "seq_is_ep_start": host(self.seq_is_ep_start)[:n_seq],
            "batch_sizes": host(self.batch_sizes)[:t_max], "t_off": host(self.t_off)[:t_max + 1],
            "gather_idx": host(self.gather_idx),
            "batch_sizes_full": host(self.batch_sizes), "t_off_full": host(self.t_off),
        }


def weight_list(weights):
    """Flat host list in the order of the C ABI: per layer W_ih, W_hh, b_ih, b_hh; then W_a, b_a, w_v, b_v."""
    out = []
    for lw in weights["layers"]:
        out += [lw["W_ih"], lw["W_hh"], lw["b_ih"], lw["b_hh"]]
    out += [weights["W_a"], weights["b_a"], weights["w_v"], weights["b_v"]]
    return [np.asarray(a, np.float32) for a in out]


def grads_to_list(grads):
    out = []
    for gl in grads["layers"]:
        out += [gl["W_ih"], gl["W_hh"], gl["b_ih"], gl["b_hh"]]
    out += [grads["W_a"], grads["b_a"], grads["w_v"], grads["b_v"]]
    return out


GRAD_NAMES = ["W_ih", "W_hh", "b_ih", "b_hh"]


def meta_to_device(meta):
    """Oracle packing metadata -> the device arrays ver_lstm_* read (padded like ver_pack_minibatch pads)."""
    M, t_max = meta["M"], meta["T_max"]
    info = np.array([meta["n_seq"], t_max, meta["K"], 0], np.int32)
    bs = np.zeros(M, np.int32)
    bs[:t_max] = meta["batch_sizes"]
    t_off = np.full(M + 1, M, np.int32)
    t_off[:t_max + 1] = meta["t_off"]
    return dev(info), dev(bs), dev(t_off)


class LstmRun:
    """One forward (+ optional backward) of the HIP LSTM on packed rows."""

    def __init__(self, ver, w, weights, x_packed, meta, h0=None, c0=None, compute=0, x_bf16=False, layer_by_layer=False):
        self.ver, self.M = ver, meta["M"]
        self.cfg = ver.lstm_cfg(w.n_layers, w.input_dim, w.hidden, w.act_dim, compute, int(x_bf16), int(layer_by_layer))
        self.w_host = weight_list(weights)
        self.w_dev = [dev(a) for a in self.w_host]
        x = torch.from_numpy(np.ascontiguousarray(x_packed)).cuda()
        self.x = x.to(torch.bfloat16) if x_bf16 else x
        self.info, self.bs, self.t_off = meta_to_device(meta)
        self.seq_cap = max(1, meta["n_seq"])
        self.h0 = dev(np.ascontiguousarray(h0, np.float32)) if h0 is not None else None
        self.c0 = dev(np.ascontiguousarray(c0, np.float32)) if c0 is not None else None
        self.ws = ver.workspace(ver.ver_lstm_workspace_bytes(self.cfg, self.M))
        self.ws.fill_(-1)
        self.head_out = torch.full((self.M, w.act_dim), float("nan"), device="cuda")
        self.value = torch.full((self.M,), float("nan"), device="cuda")

    def forward(self):
        self.ver.ver_lstm_fwd(self.cfg, self.x, self.M, self.info, self.bs, self.t_off, self.h0, self.c0,
                              self.seq_cap, self.w_dev, self.head_out, self.value, self.ws)
        torch.cuda.synchronize()
        assert self.ws[0].item() == 0, "device-side wait timed out"
        return host(self.head_out), host(self.value)

    def backward(self, d_u, d_v, want_dx=True):
        self.g_dev = [torch.full_like(t, float("nan")) for t in self.w_dev]
        self.d_x = torch.full((self.M, self.cfg.input_dim), float("nan"), device="cuda") if want_dx else None
        self.ver.ver_lstm_bwd(self.cfg, self.x, self.M, self.info, self.bs, self.t_off, self.h0, self.c0,
                              self.seq_cap, self.w_dev, dev(np.asarray(d_u, np.float32)),
                              dev(np.asarray(d_v, np.float32)), self.g_dev, self.d_x, self.ws)
        torch.cuda.synchronize()
        assert self.ws[0].item() == 0, "device-side wait timed out"
        return [host(g) for g in self.g_dev], (host(self.d_x) if want_dx else None)
