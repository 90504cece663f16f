"""Host-side checks of the C boundary that need no GPU: every function declared in
include/dqn_mi355.h is exported by the shared library and bound in Python under the same name,
and argument validation that happens before any device work returns the documented codes."""
import ctypes as C
import os
import re

import paper_2111_01264_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dqn_mi355.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\([^;{}]*\)\s*;", text)))


def test_header_exports_and_binding_agree():
    names = declared_functions()
    assert {"dqn_act", "replay_push", "replay_sample_gather", "dqn_train_step", "dqn_sync_target"} <= set(names)
    lib = C.CDLL(P.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), "library does not export " + n
        assert n in P.EXPORTS, "binding lacks " + n
        assert callable(getattr(P, n))
    assert sorted(P.EXPORTS) == names


def test_config_struct_matches_header_size():
    # 6 int32 + 5 float + uint64 (8-byte aligned) = 24 + 20 + 4 pad + 8
    assert C.sizeof(P.dqn_config) == 56


def test_validation_errors_before_device_work():
    lib = C.CDLL(P.LIB_PATH)
    lib.dqn_last_error.restype = C.c_char_p
    out = C.c_void_p()
    assert lib.dqn_create(None, None, None, C.byref(out)) == P.DQN_EINVAL
    assert b"config is null" in lib.dqn_last_error()
    cfg = P.dqn_config()
    cfg.num_actions = 0
    assert lib.dqn_create(C.byref(cfg), None, None, C.byref(out)) == P.DQN_EINVAL
    assert lib.dqn_create(C.byref(cfg), None, None, None) == P.DQN_EINVAL
    lib.replay_create.argtypes = P.EXPORTS["replay_create"][1]
    assert lib.replay_create(100, 0, 10, 1, None, None, C.byref(out)) == P.DQN_EINVAL
    assert lib.replay_create(100, 3, 10, 1, None, None, C.byref(out)) == P.DQN_EINVAL      # 100 % 3 != 0
    assert lib.replay_create(100, 4, 26, 1, None, None, C.byref(out)) == P.DQN_EINVAL      # staging > lane
    assert lib.dqn_act(None, None, 1, C.c_float(0.1), 0, 1, None, None) == P.DQN_EINVAL
    assert lib.dqn_train_step(None, None, None, None, None, None, 1, None) == P.DQN_EINVAL
    assert lib.replay_push(None, 0, None, None, None, None, 1) == P.DQN_EINVAL
    assert lib.dqn_destroy(None) == P.DQN_OK and lib.replay_destroy(None) == P.DQN_OK
    assert lib.dqn_alg1_create(None, None, None, C.byref(out)) == P.DQN_EINVAL
    lib.dqn_alg1_run.argtypes = P.EXPORTS["dqn_alg1_run"][1]
    assert lib.dqn_alg1_run(None, 0) == P.DQN_EINVAL and lib.dqn_alg1_flush(None) == P.DQN_EINVAL
    assert lib.dqn_alg1_destroy(None) == P.DQN_OK
    assert lib.dqn_envs_create(None, None, 1, C.byref(out)) == P.DQN_EINVAL
    assert lib.dqn_envs_observe(None) == P.DQN_EINVAL and lib.dqn_envs_destroy(None) == P.DQN_OK


def test_alg1_config_struct_matches_header_size():
    # 4 int32 + float + 3 uint32 + 2 int32 + 2 uint32 + uint64
    assert C.sizeof(P.dqn_alg1_config) == 56
