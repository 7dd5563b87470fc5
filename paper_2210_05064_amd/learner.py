"""One PPO update of the VER learner as a sequence of C-ABI calls.

Buffer management and argument marshalling only: every step of the update
(advantages, minibatch packing, LSTM forward, PPO loss, LSTM backward, optimiser
step) runs in the HIP library.  Used by the benchmark, the smoke check and the end-to-end
tests.  Nothing here synchronises the stream.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as ver
from .workloads import Workload


def _dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


class Learner:
    """Device-resident rollout + weights + every scratch buffer of one update."""

    def __init__(self, rollout: dict, *, compute: int | None = None, x_bf16: bool | None = None,
                 want_dx: bool = False, minibatches: int | None = None, adam_total_steps: int | None = None,
                 adam: dict | None = None, max_is: float | None = None, learned_entropy: dict | None = None,
                 arrival: tuple | None = None, want_grad_norm: bool = False, layer_by_layer: bool = False):
        """layer_by_layer: the library's diagnostic switch (two-layer networks run one launch per layer).
        want_grad_norm: have every optimiser step report the global gradient norm (always on with clipping).
        arrival: (arr_env, arr_t, csr_of_arrival) of workloads.arrival_order: the rollout is then held as the
        linear collection buffer (steps in arrival order) and every update starts by bucketing it by environment
        on the GPU (ver_ingest + one gather per field); None = the rollout is given environment-major.
        learned_entropy: dict alpha0, lower, upper, target, sign: the entropy coefficient is a device-resident
        parameter, the last tensor of the optimiser step, kept inside [lower, upper]; None = fixed coefficient.
        max_is: truncation of the per-step importance weight; None = unweighted loss.
        adam_total_steps: length of the cosine schedule in optimiser steps; None = no optimiser (gradients only).
        adam: overrides of the optimiser's hyper-parameters (fields of ver_adam_cfg)."""
        w: Workload = rollout["workload"]
        self.w = w
        self.S, self.N = rollout["S"], rollout["N"]
        self.B = minibatches or w.minibatches
        self.M = self.S // self.B
        self.compute = int(w.bf16) if compute is None else compute
        self.x_bf16 = bool(self.compute) if x_bf16 is None else x_bf16
        S, M, H, nl, A, D = self.S, self.M, w.hidden, w.n_layers, w.act_dim, w.input_dim
        f32 = dict(dtype=torch.float32, device="cuda")
        i32 = dict(dtype=torch.int32, device="cuda")
        # rollout buffer
        self.rewards, self.values = _dev(rollout["rewards"]), _dev(rollout["values"])
        self.dones, self.last_values = _dev(rollout["dones"]), _dev(rollout["last_values"])
        self.env_off = _dev(rollout["env_off"])
        self.env_started = _dev(rollout["env_started_episode"])
        self.obs, self.actions = _dev(rollout["obs"]), _dev(rollout["actions"])
        self.seq_key = _dev(rollout["seq_key"])
        self.rnn_h = _dev(rollout["rnn_h"]) if "rnn_h" in rollout else None
        self.rnn_c = _dev(rollout["rnn_c"]) if "rnn_c" in rollout else None
        self.logp_old = torch.zeros(S, **f32)
        self.arrival = None
        if arrival is not None:
            arr_env, arr_t, csr_of_arrival = arrival
            self.csr_of_arrival = torch.from_numpy(np.asarray(csr_of_arrival, np.int64)).cuda()
            # (arrival-order source, environment-major destination, leading dimensions that are not the step)
            pairs = [(self.rewards, 0), (self.values, 0), (self.dones, 0), (self.obs, 0), (self.actions, 0),
                     (self.seq_key, 1), (self.logp_old, 0)]
            pairs += [(t, 1) for t in (self.rnn_h, self.rnn_c) if t is not None]
            self.arrival = []
            for dst, lead in pairs:
                src = dst.index_select(lead, self.csr_of_arrival).contiguous()
                dst.fill_(0)                   # the environment-major copy is produced by ingest()
                self.arrival.append((src, dst, lead))
            self.arr_env, self.arr_t = _dev(np.asarray(arr_env, np.int32)), _dev(np.asarray(arr_t, np.int32))
            self.env_off.fill_(0)
            self.order = torch.empty(S, **i32)
            self.ingest_info = torch.zeros(4, **i32)
            self.ws_ingest = ver.workspace(ver.ver_ingest_workspace_bytes(self.N, S))
        self.adv, self.ret = torch.empty(S, **f32), torch.empty(S, **f32)
        self.max_is = max_is
        self.is_w = torch.empty(S, **f32) if max_is is not None else None
        # weights, gradients
        wt = rollout["weights"]
        flat = []
        for lw in wt["layers"]:
            flat += [lw["W_ih"], lw["W_hh"], lw["b_ih"], lw["b_hh"]]
        flat += [wt["W_a"], wt["b_a"], wt["w_v"], wt["b_v"]]
        self.weights = [_dev(np.asarray(a, np.float32)) for a in flat]
        self.grads = [torch.empty_like(t) for t in self.weights]
        self.log_std = _dev(np.asarray(wt["log_std"], np.float32))
        self.d_log_std = torch.empty(A, **f32)
        # packed minibatch: one set of index arrays (and index workspace) per minibatch of an update, so that one
        # launch can index all of them before the first minibatch runs; set 0 also serves single pack() calls
        self.index_sets = [self._index_set() for _ in range(w.epochs * self.B)]
        self._use_index_set(0)
        self.x_packed = torch.empty((M, D), dtype=torch.bfloat16 if self.x_bf16 else torch.float32, device="cuda")
        self.act_packed = torch.empty((M,) + tuple(self.actions.shape[1:]), dtype=self.actions.dtype, device="cuda")
        self.logp_old_p, self.adv_p, self.ret_p = (torch.empty(M, **f32) for _ in range(3))
        self.is_w_p = torch.empty(M, **f32) if max_is is not None else None
        self.seq_cap = M
        self.h0 = torch.empty((nl, M, H), **f32) if self.rnn_h is not None else None
        self.c0 = torch.empty((nl, M, H), **f32) if self.rnn_c is not None else None
        # network outputs, loss
        self.head_out, self.value = torch.empty((M, A), **f32), torch.empty(M, **f32)
        self.d_head, self.d_value = torch.empty((M, A), **f32), torch.empty(M, **f32)
        self.d_x = torch.empty((M, D), **f32) if want_dx else None
        self.scalars = torch.zeros(6, **f32)
        self.learned_entropy = learned_entropy
        if learned_entropy is not None:
            self.alpha = torch.full((1,), float(learned_entropy["alpha0"]), **f32)
            self.d_alpha = torch.zeros(1, **f32)
        # configuration structs and workspaces
        self.lstm_cfg = ver.lstm_cfg(nl, D, H, A, self.compute, int(self.x_bf16), int(layer_by_layer))
        self.ppo_cfg = ver.ppo_cfg(w.clip, w.value_coef, w.entropy_coef, w.dist, A)
        self.ws_gae = ver.workspace(ver.ver_gae_workspace_bytes(S))
        n = ver.ver_lstm_workspace_bytes(self.lstm_cfg, M)
        if n == 0:
            raise ver.VerError(-3)
        self.ws_lstm = ver.workspace(n)
        self.ws_loss = ver.workspace(ver.ver_ppo_loss_workspace_bytes(M, A))
        self.act_bytes = int(self.actions[0].numel() * self.actions.element_size())
        # optimiser: Adam state for every weight tensor (and log_std for Gaussian policies)
        self.adam_cfg = None
        if adam_total_steps is not None:
            self.adam_cfg = ver.adam_cfg(total_steps=adam_total_steps, **(adam or {}))
            self.opt_params = self.weights + ([self.log_std] if w.dist == 1 else [])
            self.opt_grads = self.grads + ([self.d_log_std] if w.dist == 1 else [])
            self.opt_lower = self.opt_upper = None
            if learned_entropy is not None:
                inf = float("inf")
                self.opt_lower = [-inf] * len(self.opt_params) + [float(learned_entropy["lower"])]
                self.opt_upper = [inf] * len(self.opt_params) + [float(learned_entropy["upper"])]
                self.opt_params = self.opt_params + [self.alpha]
                self.opt_grads = self.opt_grads + [self.d_alpha]
            self.exp_avg = [torch.zeros_like(t) for t in self.opt_params]
            self.exp_avg_sq = [torch.zeros_like(t) for t in self.opt_params]
            self.grad_norm = torch.zeros(1, **f32)
            self.want_grad_norm = want_grad_norm or self.adam_cfg.max_grad_norm > 0
            self.ws_adam = ver.workspace(ver.ver_adam_workspace_bytes())
            self.opt_steps = 0

    def _index_set(self) -> dict:
        M = self.M
        i32 = dict(dtype=torch.int32, device="cuda")
        return dict(info=torch.zeros(4, **i32), seq_first=torch.empty(M, **i32), seq_len=torch.empty(M, **i32),
                    seq_eps=torch.empty(M, dtype=torch.uint8, device="cuda"), batch_sizes=torch.empty(M, **i32),
                    t_off=torch.empty(M + 1, **i32), gather_idx=torch.empty(M, **i32),
                    ws_pack=ver.workspace(ver.ver_pack_workspace_bytes(self.N, self.S, self.B)))

    def _use_index_set(self, k: int):
        for name, t in self.index_sets[k].items():
            setattr(self, name, t)

    def _pack_args(self, epoch: int, b: int, index_ready: int):
        return ver.pack_args(
            dones=self.dones, env_off=self.env_off, env_started_episode=self.env_started,
            seq_key=self.seq_key[epoch], N=self.N, S=self.S, B=self.B, b=b,
            info=self.info, seq_first=self.seq_first, seq_len=self.seq_len, seq_is_ep_start=self.seq_eps,
            batch_sizes=self.batch_sizes, t_off=self.t_off, gather_idx=self.gather_idx,
            obs=self.obs, D=self.w.input_dim, obs_packed=self.x_packed, obs_packed_bf16=int(self.x_bf16),
            actions=self.actions, act_bytes=self.act_bytes, actions_packed=self.act_packed,
            logp_old=self.logp_old, adv=self.adv, ret=self.ret, is_weight=self.is_w,
            logp_old_packed=self.logp_old_p, adv_packed=self.adv_p, ret_packed=self.ret_p,
            is_weight_packed=self.is_w_p,
            rnn_h=self.rnn_h, rnn_c=self.rnn_c, n_layers=self.w.n_layers, H=self.w.hidden,
            seq_cap=self.seq_cap, h0=self.h0, c0=self.c0, workspace=self.ws_pack, index_ready=index_ready)

    # -- the entry points, in the order of the learning phase ---------------------
    def set_logp_old(self, flat: torch.Tensor):
        """Old log-probabilities, given environment-major (stored in arrival order when the buffer is)."""
        self.logp_old.copy_(flat)
        if self.arrival is not None:
            for src, dst, _ in self.arrival:
                if dst is self.logp_old:
                    src.copy_(flat[self.csr_of_arrival])

    def ingest(self):
        ver.ver_ingest(self.arr_env, self.arr_t, self.N, self.S, self.env_off, self.order, self.ingest_info, self.ws_ingest)
        pairs = []
        for src, dst, lead in self.arrival:
            if lead == 0:
                pairs.append((src, dst))
            else:
                pairs += [(src[j], dst[j]) for j in range(src.shape[0])]
        ver.ver_ingest_gather_batch(self.order, self.S, pairs)   # every per-step field in one launch

    def gae(self):
        ver.ver_gae(self.rewards, self.values, self.dones, self.last_values, self.env_off, self.N, self.S,
                    self.w.gamma, self.w.lam, self.adv, self.ret, self.ws_gae)

    def importance_weights(self):
        ver.ver_is_weight(self.env_off, self.N, self.S, self.max_is, self.is_w)

    def pack(self, epoch: int, b: int, index_ready: bool = False):
        """Index + gathers of one minibatch into the current index set (index_ready: gathers only)."""
        a = self._pack_args(epoch, b, int(index_ready))
        ver._check(ver.lib.ver_pack_minibatch(a, ver._stream()))

    def index_all(self):
        """The index arrays of every minibatch of the update (epochs x minibatches) in one launch."""
        blocks = []
        for e in range(self.w.epochs):
            for b in range(self.B):
                self._use_index_set(e * self.B + b)
                blocks.append(self._pack_args(e, b, 0))
        self._use_index_set(0)
        ver.ver_pack_index_batch(blocks)

    def forward(self):
        ver.ver_lstm_fwd(self.lstm_cfg, self.x_packed, self.M, self.info, self.batch_sizes, self.t_off,
                         self.h0, self.c0, self.seq_cap, self.weights, self.head_out, self.value, self.ws_lstm)

    def loss(self):
        le = self.learned_entropy
        if le is not None:
            ver.ver_ppo_loss_learned_entropy(
                self.ppo_cfg, self.M, self.head_out, self.value, self.log_std if self.w.dist == 1 else None,
                self.act_packed, self.logp_old_p, self.adv_p, self.ret_p, self.is_w_p, self.alpha,
                float(le.get("target", 0.0)), float(le.get("sign", 1.0)), self.scalars, self.d_head, self.d_value,
                self.d_log_std if self.w.dist == 1 else None, self.d_alpha, self.ws_loss)
            return
        ver.ver_ppo_loss(self.ppo_cfg, self.M, self.head_out, self.value,
                         self.log_std if self.w.dist == 1 else None, self.act_packed, self.logp_old_p,
                         self.adv_p, self.ret_p, self.is_w_p, self.scalars, self.d_head, self.d_value,
                         self.d_log_std if self.w.dist == 1 else None, self.ws_loss)

    def backward(self):
        ver.ver_lstm_bwd(self.lstm_cfg, self.x_packed, self.M, self.info, self.batch_sizes, self.t_off,
                         self.h0, self.c0, self.seq_cap, self.weights, self.d_head, self.d_value, self.grads,
                         self.d_x, self.ws_lstm)

    def optimizer_step(self):
        ver.ver_adam_step_bounded(self.adam_cfg, self.opt_params, self.opt_grads, self.exp_avg, self.exp_avg_sq,
                                  self.opt_lower, self.opt_upper, self.opt_steps,
                                  self.grad_norm if self.want_grad_norm else None, self.ws_adam)
        self.opt_steps += 1

    def minibatch(self, epoch: int, b: int, index_ready: bool = False):
        self.pack(epoch, b, index_ready)
        self.forward()
        self.loss()
        self.backward()
        if self.adam_cfg is not None:
            self.optimizer_step()

    def update(self, on_minibatch=None):
        """One PPO update: advantages (and importance weights) once, then epochs x minibatches."""
        if self.arrival is not None:
            self.ingest()
        self.gae()
        if self.max_is is not None:
            self.importance_weights()
        self.index_all()
        for e in range(self.w.epochs):
            for b in range(self.B):
                self._use_index_set(e * self.B + b)
                self.minibatch(e, b, index_ready=True)
                if on_minibatch is not None:
                    on_minibatch(e, b)

    def lstm_timed_out(self) -> bool:
        """A bounded device-side wait of the LSTM time loops gave up (synchronises)."""
        return bool(self.ws_lstm[0].item() != 0)

    def gae_timed_out(self) -> bool:
        """A bounded look-back wait of the advantage scan gave up (synchronises)."""
        return bool(self.ws_gae[1].item() != 0)
