"""The built library loads without a GPU and exports every entry point that
include/ver.h declares; host-only queries and argument checks behave.  CPU only
(no kernel is launched)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2210_05064_amd", "libver.so")
HEADER = os.path.join(ROOT, "include", "ver.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2210_05064_amd import build
        build.build(verbose=False)
    return C.CDLL(LIB)


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(ver_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"ver_gae", "ver_pack_minibatch", "ver_lstm_fwd", "ver_lstm_bwd", "ver_ppo_loss"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in ver.h but not exported"


def test_status_strings(lib):
    lib.ver_status_string.restype = C.c_char_p
    seen = {lib.ver_status_string(c).decode() for c in (0, -1, -2, -3, -4, -5)}
    assert len(seen) == 6 and lib.ver_status_string(-99)


def test_workspace_queries_are_host_only(lib):
    lib.ver_gae_workspace_bytes.restype = C.c_size_t
    lib.ver_pack_workspace_bytes.restype = C.c_size_t
    lib.ver_ppo_loss_workspace_bytes.restype = C.c_size_t
    lib.ver_lstm_workspace_bytes.restype = C.c_size_t
    assert lib.ver_gae_workspace_bytes(32768) >= 256 + 16 * 28
    assert lib.ver_gae_workspace_bytes(-1) == 0
    assert lib.ver_pack_workspace_bytes(256, 32768, 4) >= 21 * 32768
    assert lib.ver_ppo_loss_workspace_bytes(8192, 11) > 0

    class Cfg(C.Structure):
        _fields_ = [(n, C.c_int32) for n in ("n_layers", "input_dim", "hidden", "act_dim", "compute", "x_bf16",
                                                 "layer_by_layer")]
    big = lib.ver_lstm_workspace_bytes(C.byref(Cfg(2, 1044, 1024, 11, 1, 1, 0)), 8192)
    assert big > 2 * 8192 * 6 * 1024 * 4          # saved activations of two layers at least
    assert lib.ver_lstm_workspace_bytes(C.byref(Cfg(2, 1044, 1024, 11, 0, 0, 0)), 8192) == 0   # fp32 needs hidden <= 512
    assert lib.ver_lstm_workspace_bytes(C.byref(Cfg(2, 1044, 1000, 11, 1, 1, 0)), 8192) == 0


def test_argument_checks_precede_any_gpu_work(lib):
    lib.ver_gae.argtypes = [C.c_void_p] * 5 + [C.c_int32, C.c_int32, C.c_float, C.c_float] + [C.c_void_p] * 3 + \
        [C.c_size_t, C.c_void_p]
    assert lib.ver_gae(None, None, None, None, None, 1, -5, 0.99, 0.95, None, None, None, 0, None) == -1
    assert lib.ver_gae(None, None, None, None, None, 1, 0, 0.99, 0.95, None, None, None, 0, None) == 0
    assert lib.ver_gae(None, None, None, None, None, 1, 8, 0.99, 0.95, None, None, None, 0, None) == -1
    lib.ver_pack_minibatch.argtypes = [C.c_void_p, C.c_void_p]
    assert lib.ver_pack_minibatch(None, None) == -1
    lib.ver_ppo_loss.argtypes = [C.c_void_p, C.c_int32] + [C.c_void_p] * 13 + [C.c_size_t, C.c_void_p]
    assert lib.ver_ppo_loss(None, 4, *([None] * 13), 0, None) == -1


def test_adam_argument_checks(lib):
    class AdamCfg(C.Structure):
        _fields_ = [("lr0", C.c_float), ("lr_final", C.c_float), ("total_steps", C.c_int64), ("beta1", C.c_float),
                    ("beta2", C.c_float), ("eps", C.c_float), ("max_grad_norm", C.c_float)]
    lib.ver_adam_workspace_bytes.restype = C.c_size_t
    assert lib.ver_adam_workspace_bytes() > 0
    lib.ver_adam_step.argtypes = [C.c_void_p, C.c_int32] + [C.c_void_p] * 5 + [C.c_int64] + [C.c_void_p] * 2 + \
        [C.c_size_t, C.c_void_p]
    ok = AdamCfg(2.5e-4, 0.0, 10, 0.9, 0.999, 1e-8, 0.0)
    empty = (C.c_void_p * 1)()
    sizes = (C.c_int64 * 1)(0)
    call = lambda cfg, n, step: lib.ver_adam_step(C.byref(cfg) if cfg else None, n, empty, empty, empty, empty, sizes, step,
                                                  None, None, 0, None)
    assert call(None, 0, 0) == -1
    assert call(ok, 0, 0) == 0                       # nothing to update
    assert call(ok, 1, 0) == 0                       # one tensor of size 0
    assert call(ok, -1, 0) == -1 and call(ok, 1000, 0) == -1 and call(ok, 1, -3) == -1
    assert call(AdamCfg(2.5e-4, 0.0, 0, 0.9, 0.999, 1e-8, 0.0), 1, 0) == -1      # no schedule length
    assert call(AdamCfg(2.5e-4, 0.0, 10, 1.0, 0.999, 1e-8, 0.0), 1, 0) == -1     # beta1 = 1
    assert call(AdamCfg(2.5e-4, 0.0, 10, 0.9, 0.999, 1e-8, 1.0), 1, 0) == -1     # clipping needs grad_norm
    sizes[0] = 8
    assert call(ok, 1, 0) == -1                      # null tensors of positive size


def test_is_weight_argument_checks(lib):
    lib.ver_is_weight.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p]
    assert lib.ver_is_weight(None, 4, 0, 1.0, None, None) == 0        # empty buffer: nothing to do
    assert lib.ver_is_weight(None, 4, 16, 1.0, None, None) == -1      # null pointers
    assert lib.ver_is_weight(None, 0, 0, 1.0, None, None) == -1       # no environments
    assert lib.ver_is_weight(None, 4, 0, 0.0, None, None) == -1       # truncation must be positive
    assert lib.ver_is_weight(None, 4, 0, float("nan"), None, None) == -1
    assert lib.ver_is_weight(None, 4, -1, 1.0, None, None) == -1


def test_learned_entropy_and_bounded_step_argument_checks(lib):
    lib.ver_ppo_loss_learned_entropy.argtypes = [C.c_void_p, C.c_int32] + [C.c_void_p] * 9 + [C.c_float, C.c_float] + \
        [C.c_void_p] * 6 + [C.c_size_t, C.c_void_p]
    one = C.c_void_p(16)      # never dereferenced: the checks below fail before any GPU work
    assert lib.ver_ppo_loss_learned_entropy(None, 4, *([None] * 9), 0.0, 1.0, *([None] * 6), 0, None) == -1
    # alpha and d_alpha present, a sign other than +1 / -1
    assert lib.ver_ppo_loss_learned_entropy(None, 4, *([None] * 8), one, 0.0, 0.5, *([None] * 4), one, None, 0, None) == -1
    # valid sign, but the remaining arguments are still checked
    assert lib.ver_ppo_loss_learned_entropy(None, 4, *([None] * 8), one, 0.0, -1.0, *([None] * 4), one, None, 0, None) == -1

    class AdamCfg(C.Structure):
        _fields_ = [("lr0", C.c_float), ("lr_final", C.c_float), ("total_steps", C.c_int64), ("beta1", C.c_float),
                    ("beta2", C.c_float), ("eps", C.c_float), ("max_grad_norm", C.c_float)]
    lib.ver_adam_step_bounded.argtypes = [C.c_void_p, C.c_int32] + [C.c_void_p] * 7 + [C.c_int64] + [C.c_void_p] * 2 + \
        [C.c_size_t, C.c_void_p]
    ok = AdamCfg(2.5e-4, 0.0, 10, 0.9, 0.999, 1e-8, 0.0)
    empty = (C.c_void_p * 1)()
    sizes = (C.c_int64 * 1)(0)
    call = lambda lo, hi: lib.ver_adam_step_bounded(C.byref(ok), 1, empty, empty, empty, empty, sizes,
                                                    (C.c_float * 1)(lo) if lo is not None else None,
                                                    (C.c_float * 1)(hi) if hi is not None else None, 0, None, None, 0, None)
    assert call(None, None) == 0 and call(1e-4, 1.0) == 0 and call(None, 1.0) == 0 and call(0.5, 0.5) == 0
    assert call(1.0, 1e-4) == -1                      # empty box
    assert call(float("nan"), 1.0) == -1 and call(0.0, float("nan")) == -1


def test_ingest_argument_checks(lib):
    lib.ver_ingest_workspace_bytes.restype = C.c_size_t
    lib.ver_ingest_workspace_bytes.argtypes = [C.c_int32, C.c_int32]
    assert lib.ver_ingest_workspace_bytes(256, 32768) >= 3 * 32768 * 4
    assert lib.ver_ingest_workspace_bytes(0, 8) == 0 and lib.ver_ingest_workspace_bytes(4, -1) == 0
    assert lib.ver_ingest_workspace_bytes(4, (1 << 24) + 1) == 0
    lib.ver_ingest.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32] + [C.c_void_p] * 4 + [C.c_size_t, C.c_void_p]
    assert lib.ver_ingest(None, None, 4, 8, None, None, None, None, 0, None) == -1
    assert lib.ver_ingest(None, None, 0, 0, None, None, None, None, 0, None) == -1
    lib.ver_ingest_dense.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    assert lib.ver_ingest_dense(4, 0, None, None, None) == -1 and lib.ver_ingest_dense(-1, 4, None, None, None) == -1
    assert lib.ver_ingest_dense(4, 4, None, None, None) == -1
    lib.ver_ingest_gather.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    assert lib.ver_ingest_gather(None, 0, None, 4, None, None) == 0        # nothing to move
    assert lib.ver_ingest_gather(None, 8, None, 4, None, None) == -1
    assert lib.ver_ingest_gather(None, 8, None, 0, None, None) == -1
    lib.ver_ingest_gather_batch.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    assert lib.ver_ingest_gather_batch(None, 0, 3, None, None, None, None) == 0     # no steps: nothing to move
    assert lib.ver_ingest_gather_batch(None, 8, 0, None, None, None, None) == 0     # no fields
    assert lib.ver_ingest_gather_batch(None, 8, 2, None, None, None, None) == -1
    assert lib.ver_ingest_gather_batch(None, 8, 25, None, None, None, None) == -1   # more than VER_INGEST_MAX_FIELDS


def test_pack_index_batch_argument_checks(lib):
    lib.ver_pack_index_batch.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    assert lib.ver_pack_index_batch(None, 0, None) == 0        # nothing to index
    assert lib.ver_pack_index_batch(None, 3, None) == -1
    assert lib.ver_pack_index_batch(None, -1, None) == -1
