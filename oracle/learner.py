"""CPU oracle: one PPO minibatch step of the VER learner, end to end.

TEST INFRASTRUCTURE ONLY.  Chains the oracle's parts in the order of the
paper's learning phase (section 2.2): advantages once per rollout, then for
every minibatch: cut it out of the randomly ordered sequences, run the
recurrent policy over each of its pieces, evaluate the PPO loss, and
back-propagate through time.  Nothing in the product path may import this
file.
"""
import numpy as np

from . import adam, entropy_coef, is_weight, lstm, pack, ppo_loss


def minibatch_step(rollout_fields, weights, meta, cfg, adv, ret, logp_old, h0=None, c0=None,
                   weight=None, want_dx=False, alpha=None):
    """One minibatch: forward, loss, backward.

    rollout_fields: dict with flat per-step "obs" [S, D] and "actions".
    meta: result of pack.pack_minibatch.  adv, ret, logp_old: flat [S].
    cfg: dict with dist, clip, value_coef, entropy_coef.  alpha: current value of the learned entropy
    coefficient (then cfg holds target_entropy and alpha_sign instead of entropy_coef), None = fixed.
    Returns dict: u, v (packed rows), scalars, d_u, d_v, grads (incl. log_std), d_x, d_alpha.
    """
    w64 = lstm.weights_f64(weights)
    gidx = meta["gather_idx"]
    fwd = lstm.minibatch_forward(rollout_fields["obs"], meta["seq_first"], meta["seq_len"], w64, h0, c0)
    u = lstm.to_packed([f[0] for f in fwd], meta["t_off"])
    v = lstm.to_packed([f[1] for f in fwd], meta["t_off"])
    rows = (cfg["dist"], u, v, w64["log_std"], pack.gather_rows(rollout_fields["actions"], gidx),
            pack.gather_rows(logp_old, gidx), pack.gather_rows(adv, gidx), pack.gather_rows(ret, gidx))
    w_rows = None if weight is None else pack.gather_rows(weight, gidx)
    d_alpha = None
    if alpha is None:
        scalars, d_u, d_v, d_log_std = ppo_loss.ppo_loss(*rows, cfg["clip"], cfg["value_coef"], cfg["entropy_coef"], w_rows)
    else:
        scalars, d_u, d_v, d_log_std, d_alpha = entropy_coef.ppo_loss_learned_entropy(
            *rows, cfg["clip"], cfg["value_coef"], alpha, cfg["target_entropy"], w_rows, cfg.get("alpha_sign", 1.0))
    grads = lstm.zero_grads(w64)
    du_pieces = lstm.from_packed(d_u, meta["t_off"], meta["seq_len"])
    dv_pieces = lstm.from_packed(d_v, meta["t_off"], meta["seq_len"])
    dx_pieces = []
    for j in range(meta["n_seq"]):
        dx_pieces.append(lstm.piece_backward(du_pieces[j], dv_pieces[j], w64, fwd[j][2], grads))
    grads["log_std"] = d_log_std
    out = {"u": u, "v": v, "scalars": scalars, "d_u": d_u, "d_v": d_v, "grads": grads, "d_alpha": d_alpha}
    if want_dx:
        out["d_x"] = lstm.to_packed(dx_pieces, meta["t_off"])
    return out


def collection_logp(rollout_fields, weights, dones, env_off, dist, env_started_episode=None,
                    rnn_h=None, rnn_c=None):
    """Log-probability of every stored action under `weights`, evaluated over
    whole sequences (what the policy assigned when the step was collected).
    Used by tests to build logp_old; returns flat [S] fp64."""
    w64 = lstm.weights_f64(weights)
    first, length, ep_start = pack.find_sequences(dones, env_off, env_started_episode)
    S = int(env_off[-1])
    logp = np.zeros(S)
    h0 = c0 = None
    if rnn_h is not None:
        h0 = pack.initial_states(rnn_h, first, ep_start)
        c0 = pack.initial_states(rnn_c, first, ep_start)
    fwd = lstm.minibatch_forward(rollout_fields["obs"], first, length, w64, h0, c0)
    for j, (f0, n) in enumerate(zip(first, length)):
        u = fwd[j][0]
        for t in range(n):
            logp[f0 + t] = ppo_loss.row_logp_entropy(dist, u[t], rollout_fields["actions"][f0 + t],
                                                     w64["log_std"])[0]
    return logp


# order of the tensors in an optimiser step: per layer W_ih, W_hh, b_ih, b_hh, then the heads, then log_std
def _flatten(weights, with_log_std):
    out = []
    for lw in weights["layers"]:
        out += [lw["W_ih"], lw["W_hh"], lw["b_ih"], lw["b_hh"]]
    out += [weights["W_a"], weights["b_a"], weights["w_v"], weights["b_v"]]
    if with_log_std:
        out.append(weights["log_std"])
    return [np.asarray(a, np.float64) for a in out]


def _unflatten(flat, like, with_log_std):
    it = iter(flat)
    w = {"layers": [{k: next(it) for k in ("W_ih", "W_hh", "b_ih", "b_hh")} for _ in like["layers"]]}
    for k in ("W_a", "b_a", "w_v", "b_v"):
        w[k] = next(it)
    w["log_std"] = next(it) if with_log_std else np.asarray(like["log_std"], np.float64)
    return w


def ppo_update(rollout, adv, ret, logp_old, cfg, opt, h0_fields=None, max_is=None, learned_entropy=None):
    """One whole PPO update with the optimiser in the loop (the paper's learning phase followed by its Adam
    step, section 2.2 and section 4 "Training"): for every epoch and minibatch, pack, forward, loss, backward,
    Adam.  rollout: dict of workloads.make_rollout; cfg: loss hyper-parameters + "epochs", "minibatches";
    opt: dict lr0, lr_final, total_steps, beta1, beta2, eps, max_grad_norm; max_is: truncation of the per-step
    importance weight of the loss (None = unweighted); learned_entropy: dict alpha0, lower, upper (cfg then
    holds target_entropy / alpha_sign): the coefficient is the last tensor of the optimiser step and is
    projected onto its bounds after every step.  Returns the final weights (fp64),
    the list of per-minibatch scalars and the gradient norms."""
    gauss = cfg["dist"] == ppo_loss.GAUSSIAN
    weights = _unflatten(_flatten(rollout["weights"], gauss), rollout["weights"], gauss)
    params = _flatten(weights, gauss)
    if learned_entropy is not None:
        params.append(np.array([learned_entropy["alpha0"]], np.float64))
    m = [np.zeros_like(p) for p in params]
    v = [np.zeros_like(p) for p in params]
    scalars, norms, k = [], [], 0
    weight = None if max_is is None else is_weight.is_weights(rollout["env_off"], max_is)
    for e in range(cfg["epochs"]):
        for b in range(cfg["minibatches"]):
            meta = pack.pack_minibatch(rollout["dones"], rollout["env_off"], rollout["seq_key"][e], cfg["minibatches"], b,
                                       rollout.get("env_started_episode"))
            h0 = c0 = None
            if "rnn_h" in rollout:
                h0 = pack.initial_states(rollout["rnn_h"], meta["seq_first"], meta["seq_is_ep_start"])
                c0 = pack.initial_states(rollout["rnn_c"], meta["seq_first"], meta["seq_is_ep_start"])
            out = minibatch_step(rollout, weights, meta, cfg, adv, ret, logp_old, h0, c0, weight=weight,
                                 alpha=None if learned_entropy is None else float(params[-1][0]))
            g = out["grads"]
            grads = []
            for lg in g["layers"]:
                grads += [lg["W_ih"], lg["W_hh"], lg["b_ih"], lg["b_hh"]]
            grads += [g["W_a"], g["b_a"], g["w_v"], g["b_v"]]
            if gauss:
                grads.append(g["log_std"])
            if learned_entropy is not None:
                grads.append(np.array([out["d_alpha"]], np.float64))
            lr = adam.cosine_lr(k, opt["total_steps"], opt["lr0"], opt["lr_final"])
            params, m, v, norm = adam.adam_step(params, grads, m, v, k + 1, lr, opt["beta1"], opt["beta2"], opt["eps"],
                                                opt["max_grad_norm"])
            if learned_entropy is not None:
                inf = np.inf
                params = adam.project(params, [-inf] * (len(params) - 1) + [learned_entropy["lower"]],
                                      [inf] * (len(params) - 1) + [learned_entropy["upper"]])
            weights = _unflatten(params, weights, gauss)
            scalars.append(out["scalars"])
            norms.append(norm)
            k += 1
    if learned_entropy is not None:
        return weights, scalars, norms, float(params[-1][0])
    return weights, scalars, norms
