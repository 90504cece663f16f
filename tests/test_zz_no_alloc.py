"""dqn_act_static (the act step for callers that cannot allocate: its intermediates live in a fixed array of the
library's device image) against dqn_act, through the C boundary: identical kernels on identical inputs, so Q rows and
actions must agree bit for bit; two calls in a row, the second on fewer states, in both precisions."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2111_01264_amd as P
from datagen import synth
from tests.gpu_util import dev, make_cfg


@pytest.mark.parametrize("precision", [P.DQN_PRECISION_FP32, P.DQN_PRECISION_BF16])
def test_act_static_equals_act_bitwise_two_calls_in_a_row(precision):
    A, seed = 18, 91
    lib = C.CDLL(P.LIB_PATH)
    for name in ("dqn_act", "dqn_act_static"):
        getattr(lib, name).argtypes = P.EXPORTS[name][1]
        getattr(lib, name).restype = C.c_int
    lib.dqn_last_error.restype = C.c_char_p
    cfg = make_cfg(A, max_envs=64, precision=precision, seed=seed)
    sa, stt = torch.cuda.Stream(), torch.cuda.Stream()
    ctx = P.dqn_create(cfg, sa, stt)
    try:
        P.dqn_set_params(ctx, P.DQN_PARAMS_ONLINE, synth.init_params(seed, A))
        P.dqn_set_params(ctx, P.DQN_PARAMS_TARGET, synth.init_params(seed + 1, A))
        for call, (W, eps, use_target) in enumerate([(P.DQN_ACT_STATIC_MAX_ENVS, 0.1, 1), (5, 0.0, 0)]):
            states = dev(synth.act_states(seed, call, W))
            out = {}
            for name in ("dqn_act", "dqn_act_static"):
                acts = torch.full((W,), -1, dtype=torch.int32, device="cuda")
                q = torch.full((W, A), float("nan"), dtype=torch.float32, device="cuda")
                torch.cuda.synchronize()
                rc = getattr(lib, name)(ctx, states.data_ptr(), W, eps, 40 + call, use_target, acts.data_ptr(), q.data_ptr())
                assert rc == P.DQN_OK, lib.dqn_last_error()
                torch.cuda.synchronize()
                out[name] = (acts.cpu().numpy(), q.cpu().numpy())
            assert np.all(np.isfinite(out["dqn_act"][1]))
            assert np.array_equal(out["dqn_act"][1], out["dqn_act_static"][1]), ("q", call)
            assert np.array_equal(out["dqn_act"][0], out["dqn_act_static"][0]), ("actions", call)
        # beyond the fixed array's capacity: refused on the host, nothing launched
        W = P.DQN_ACT_STATIC_MAX_ENVS + 1
        states = dev(synth.act_states(seed, 2, W))
        acts = torch.empty(W, dtype=torch.int32, device="cuda")
        rc = lib.dqn_act_static(ctx, states.data_ptr(), W, 0.1, 0, 1, acts.data_ptr(), None)
        assert rc == P.DQN_EINVAL and b"fixed array" in lib.dqn_last_error()
    finally:
        P.dqn_destroy(ctx)
