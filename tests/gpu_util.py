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
