"""ver_pack_minibatch against the CPU oracle: every integer output bit-exact,
gathered fields bit-exact copies."""
import numpy as np
import pytest
import torch

from oracle import pack as opack
from paper_2210_05064_amd import workloads as wl
from tests.gpu_util import PackOut, dev, host

pytestmark = pytest.mark.gpu


def run_pack(ver, dones, off, key, B, b, eps=None, fields=None, bf16=False):
    N, S = len(off) - 1, int(off[-1])
    M = S // B
    f = fields or {}
    D = f["obs"].shape[1] if "obs" in f else 0
    nl, H = (f["rnn_h"].shape[0], f["rnn_h"].shape[2]) if "rnn_h" in f else (0, 0)
    act = f.get("actions")
    out = PackOut(M, D, act.shape[1:] if act is not None else (), torch.float32 if (act is not None and act.dtype == np.float32) else torch.int32,
                  nl, H, bf16)
    ws = ver.workspace(ver.ver_pack_workspace_bytes(N, S, B))
    ws.fill_(-1)
    kw = dict(dones=dev(dones), env_off=dev(np.asarray(off, np.int32)), seq_key=dev(key), N=N, S=S, B=B, b=b,
              env_started_episode=dev(eps) if eps is not None else None,
              info=out.info, seq_first=out.seq_first, seq_len=out.seq_len, seq_is_ep_start=out.seq_is_ep_start,
              batch_sizes=out.batch_sizes, t_off=out.t_off, gather_idx=out.gather_idx, workspace=ws)
    if "obs" in f:
        kw.update(obs=dev(f["obs"]), D=D, obs_packed=out.obs_packed, obs_packed_bf16=int(bf16))
    if act is not None:
        kw.update(actions=dev(act), act_bytes=act[0].nbytes if act.ndim > 1 else act.itemsize,
                  actions_packed=out.actions_packed)
    for k in ("logp_old", "adv", "ret", "is_weight"):
        if k in f:
            kw[k] = dev(f[k])
            kw[k + "_packed"] = getattr(out, k + "_packed")
    if "rnn_h" in f:
        kw.update(rnn_h=dev(f["rnn_h"]), rnn_c=dev(f["rnn_c"]), n_layers=nl, H=H, seq_cap=M, h0=out.h0, c0=out.c0)
    ver.ver_pack_minibatch(**kw)
    torch.cuda.synchronize()
    return out


def compare_meta(got, ref):
    assert got["K"] == ref["K"] and got["n_seq"] == ref["n_seq"] and got["T_max"] == ref["T_max"]
    for k in ("seq_first", "seq_len", "seq_is_ep_start", "batch_sizes", "t_off", "gather_idx"):
        assert np.array_equal(got[k], ref[k]), k
    M, t_max = ref["M"], ref["T_max"]
    assert np.all(got["batch_sizes_full"][t_max:] == 0)
    assert np.all(got["t_off_full"][t_max:] == M)


@pytest.mark.parametrize("name", ["tiny", "nav", "manip", "large", "max"])
def test_workload_shapes_all_minibatches(ver, name):
    w = wl.WORKLOADS[name]
    ro = wl.make_rollout(wl.scaled(w, input_dim=8, hidden=64), seed=5, with_states=False)
    covered = []
    for b in range(w.minibatches):
        out = run_pack(ver, ro["dones"], ro["env_off"], ro["seq_key"][-1], w.minibatches, b, ro["env_started_episode"])
        ref = opack.pack_minibatch(ro["dones"], ro["env_off"], ro["seq_key"][-1], w.minibatches, b,
                                   ro["env_started_episode"])
        compare_meta(out.meta(), ref)
        covered += ref["gather_idx"].tolist()
    assert sorted(covered) == list(range(ro["S"]))


@pytest.mark.parametrize("seed,n_envs,max_len,p_done,B", [
    (0, 6, 40, 0.12, 3), (1, 1, 4096, 0.0, 4), (2, 3, 3000, 1.0, 2), (3, 50, 120, 0.3, 5),
    (4, 9, 700, 0.004, 1), (5, 2, 1, 0.0, 1), (6, 1200, 4, 0.2, 2)])
def test_ragged_edge_cases(ver, seed, n_envs, max_len, p_done, B):
    """Empty environments, one environment owning everything (K = 1, split by
    cuts), every step an episode end (K = S > 1024), many tiny environments."""
    rng = np.random.default_rng(seed)
    L = rng.integers(0 if n_envs > 2 else 1, max_len + 1, size=n_envs)
    L[-1] += (-int(L.sum())) % B
    if L.sum() == 0:
        L[-1] = B
    off = np.concatenate([[0], np.cumsum(L)]).astype(np.int32)
    S = int(off[-1])
    dones = (rng.random(S) < p_done).astype(np.uint8)
    key = rng.integers(0, 2 ** 32, size=S, dtype=np.uint64).astype(np.uint32)
    if seed == 3:
        key[:] = key % 3          # many equal keys: the id tie-break decides
    eps = (rng.random(n_envs) < 0.5).astype(np.uint8)
    for b in range(B):
        out = run_pack(ver, dones, off, key, B, b, eps)
        compare_meta(out.meta(), opack.pack_minibatch(dones, off, key, B, b, eps))


@pytest.mark.parametrize("budget,n_envs", [(512, 8), (1 << 17, 700)])
@pytest.mark.parametrize("bf16", [False, True])
def test_gathered_fields(ver, bf16, budget, n_envs):
    """Every gathered field of both minibatches; 2 x 256 rows, and 2 x 65536 rows (from there on a workgroup of the
    gather kernel takes 8 rows instead of 4)."""
    w = wl.scaled(wl.WORKLOADS["manip"], input_dim=36, hidden=64, budget=budget, n_envs=n_envs)
    ro = wl.make_rollout(w, seed=9)
    rng = np.random.default_rng(0)
    fields = dict(obs=ro["obs"], actions=ro["actions"], logp_old=rng.standard_normal(ro["S"]).astype(np.float32),
                  adv=rng.standard_normal(ro["S"]).astype(np.float32),
                  ret=rng.standard_normal(ro["S"]).astype(np.float32),
                  is_weight=rng.random(ro["S"]).astype(np.float32), rnn_h=ro["rnn_h"], rnn_c=ro["rnn_c"])
    for b in range(2):
        out = run_pack(ver, ro["dones"], ro["env_off"], ro["seq_key"][0], 2, b, ro["env_started_episode"], fields, bf16)
        ref = opack.pack_minibatch(ro["dones"], ro["env_off"], ro["seq_key"][0], 2, b, ro["env_started_episode"])
        compare_meta(out.meta(), ref)
        g = ref["gather_idx"]
        if bf16:
            expect = torch.from_numpy(opack.gather_rows(ro["obs"], g)).to(torch.bfloat16)   # round to nearest even
            assert torch.equal(out.obs_packed.cpu(), expect)
        else:
            assert np.array_equal(host(out.obs_packed), opack.gather_rows(ro["obs"], g))
        assert np.array_equal(host(out.actions_packed), opack.gather_rows(ro["actions"], g))
        for k in ("logp_old", "adv", "ret", "is_weight"):
            assert np.array_equal(host(getattr(out, k + "_packed")), opack.gather_rows(fields[k], g))
        n = ref["n_seq"]
        assert np.array_equal(host(out.h0)[:, :n], opack.initial_states(ro["rnn_h"], ref["seq_first"], ref["seq_is_ep_start"]))
        assert np.array_equal(host(out.c0)[:, :n], opack.initial_states(ro["rnn_c"], ref["seq_first"], ref["seq_is_ep_start"]))
        assert np.all(np.isnan(host(out.h0)[:, n:]))       # rows beyond n_seq untouched


def test_categorical_actions_and_odd_width(ver):
    """int32 actions, D not a multiple of 4 (scalar copy path)."""
    w = wl.scaled(wl.WORKLOADS["nav"], input_dim=7, hidden=64, budget=256, n_envs=5)
    ro = wl.make_rollout(w, seed=2, with_states=False)
    out = run_pack(ver, ro["dones"], ro["env_off"], ro["seq_key"][0], 2, 1, None, dict(obs=ro["obs"], actions=ro["actions"]))
    ref = opack.pack_minibatch(ro["dones"], ro["env_off"], ro["seq_key"][0], 2, 1)
    compare_meta(out.meta(), ref)
    assert np.array_equal(host(out.obs_packed), ro["obs"][ref["gather_idx"]])
    assert np.array_equal(host(out.actions_packed), ro["actions"][ref["gather_idx"]])


def test_argument_errors(ver):
    off = np.array([0, 7], np.int32)
    d = np.zeros(7, np.uint8)
    key = np.zeros(7, np.uint32)
    with pytest.raises(ver.VerError) as e:
        run_pack(ver, d, off, key, 2, 0)           # 2 does not divide 7
    assert e.value.status == -1
    off = np.array([0, 8], np.int32)
    d, key = np.zeros(8, np.uint8), np.zeros(8, np.uint32)
    with pytest.raises(ver.VerError):
        run_pack(ver, d, off, key, 2, 2)           # b out of range


@pytest.mark.parametrize("name", ["tiny", "nav", "large", "max"])
def test_index_batch_all_minibatches_in_one_launch(ver, name):
    """ver_pack_index_batch: every (epoch, minibatch) of an update indexed by one launch, each into its own
    outputs; then ver_pack_minibatch with index_ready does only the gathers.  Everything bit-exact against the
    oracle's per-minibatch result."""
    w = wl.scaled(wl.WORKLOADS[name], hidden=64, input_dim=12)
    ro = wl.make_rollout(w, seed=21, with_states=False)
    N, S, B, E = ro["N"], ro["S"], w.minibatches, w.epochs
    M = S // B
    d_dones, d_off, d_eps = dev(ro["dones"]), dev(ro["env_off"]), dev(ro["env_started_episode"])
    d_obs = dev(ro["obs"])
    keys = [dev(ro["seq_key"][e]) for e in range(E)]
    outs, blocks, wss = [], [], []
    for e in range(E):
        for b in range(B):
            out = PackOut(M, 12)
            ws = ver.workspace(ver.ver_pack_workspace_bytes(N, S, B))
            ws.fill_(-1)
            kw = dict(dones=d_dones, env_off=d_off, env_started_episode=d_eps, seq_key=keys[e], N=N, S=S, B=B, b=b,
                      info=out.info, seq_first=out.seq_first, seq_len=out.seq_len, seq_is_ep_start=out.seq_is_ep_start,
                      batch_sizes=out.batch_sizes, t_off=out.t_off, gather_idx=out.gather_idx, workspace=ws)
            outs.append((out, kw)); wss.append(ws)
            blocks.append(ver.pack_args(**kw))
    ver.ver_pack_index_batch(blocks)
    torch.cuda.synchronize()
    for i, (out, kw) in enumerate(outs):
        e, b = divmod(i, B)
        ref = opack.pack_minibatch(ro["dones"], ro["env_off"], ro["seq_key"][e], B, b, ro["env_started_episode"])
        got = out.meta()
        assert np.all(host(out.gather_idx) == -7), "the index launch must not touch gather_idx"
        got["gather_idx"] = ref["gather_idx"]            # written by the gather call below
        compare_meta(got, ref)
        out.info_before = host(out.info).copy()
        ver.ver_pack_minibatch(obs=d_obs, D=12, obs_packed=out.obs_packed, index_ready=1, **kw)
        torch.cuda.synchronize()
        compare_meta(out.meta(), ref)
        assert np.array_equal(host(out.obs_packed), opack.gather_rows(ro["obs"], ref["gather_idx"]))


def test_index_batch_argument_errors(ver):
    w = wl.scaled(wl.WORKLOADS["tiny"], hidden=64, input_dim=8)
    ro = wl.make_rollout(w, seed=1, with_states=False)
    N, S = ro["N"], ro["S"]
    out, out2 = PackOut(S), PackOut(S)
    ws, ws2 = (ver.workspace(ver.ver_pack_workspace_bytes(N, S, 1)) for _ in range(2))
    base = dict(dones=dev(ro["dones"]), env_off=dev(ro["env_off"]), seq_key=dev(ro["seq_key"][0]), N=N, S=S, B=1, b=0)
    outs = lambda o: dict(info=o.info, seq_first=o.seq_first, seq_len=o.seq_len, seq_is_ep_start=o.seq_is_ep_start,
                          batch_sizes=o.batch_sizes, t_off=o.t_off, gather_idx=o.gather_idx)
    a = ver.pack_args(workspace=ws, **base, **outs(out))
    ver.ver_pack_index_batch([])                                              # nothing to do
    ver.ver_pack_index_batch([a, ver.pack_args(workspace=ws2, **base, **outs(out2))])
    with pytest.raises(ver.VerError):
        ver.ver_pack_index_batch([a, ver.pack_args(workspace=ws, **base, **outs(out2))])      # shared workspace
    with pytest.raises(ver.VerError):
        ver.ver_pack_index_batch([a, ver.pack_args(workspace=ws2, **base, **outs(out))])      # shared outputs
    with pytest.raises(ver.VerError):
        ver.ver_pack_index_batch([a, ver.pack_args(workspace=ws2, **dict(base, dones=dev(ro["dones"])), **outs(out2))])  # another rollout
    torch.cuda.synchronize()
