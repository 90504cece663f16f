"""ctypes binding of libdqn_mi355.so: argument marshalling only.

Every function has the name and argument order of its C declaration in include/dqn_mi355.h.
Device buffers are torch tensors (their data_ptr() is passed), streams are torch.cuda.Stream
objects (their cuda_stream handle is passed) or None for the default stream.  A non-zero return
code raises DqnError with the library's message.  There is no fallback: if the shared library is
missing, importing this module fails.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  -- imported first on purpose: the library must bind to the HIP runtime
              # that PyTorch has loaded, so that tensors, streams and kernels share one runtime

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdqn_mi355.so")

DQN_OK, DQN_EINVAL, DQN_EHIP, DQN_ENOMEM, DQN_ESTATE = 0, -1, -2, -3, -4
DQN_PRECISION_FP32, DQN_PRECISION_BF16 = 0, 1
DQN_ACT_STATIC_MAX_ENVS = 32
DQN_PARAMS_ONLINE, DQN_PARAMS_TARGET, DQN_PARAMS_RMS_V, DQN_PARAMS_RMS_M, DQN_PARAMS_GRAD = range(5)


class dqn_alg1_config(C.Structure):
    _fields_ = [
        ("W", C.c_int32), ("C", C.c_int32), ("F", C.c_int32), ("B", C.c_int32), ("epsilon", C.c_float),
        ("t_reward_neg", C.c_uint32), ("t_reward_pos", C.c_uint32), ("t_term", C.c_uint32),
        ("concurrent", C.c_int32), ("synchronized", C.c_int32), ("env_step_ns", C.c_uint32), ("reserved", C.c_uint32),
        ("env_seed", C.c_uint64),
    ]


class DqnError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("dqn_mi355 error %d: %s" % (code, message))
        self.code = code


class dqn_config(C.Structure):
    _fields_ = [
        ("num_actions", C.c_int32), ("max_batch", C.c_int32), ("max_envs", C.c_int32),
        ("precision", C.c_int32), ("double_dqn", C.c_int32), ("centered", C.c_int32),
        ("gamma", C.c_float), ("huber_delta", C.c_float), ("lr", C.c_float),
        ("rms_alpha", C.c_float), ("rms_eps", C.c_float), ("seed", C.c_uint64),
    ]


EXPORTS = {
    "dqn_create": (C.c_int, [C.POINTER(dqn_config), C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]),
    "dqn_destroy": (C.c_int, [C.c_void_p]),
    "dqn_num_params": (C.c_size_t, [C.c_void_p]),
    "dqn_set_params": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_size_t]),
    "dqn_get_params": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_size_t]),
    "dqn_act": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_uint64, C.c_int32,
                          C.c_void_p, C.c_void_p]),
    "dqn_act_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_uint64, C.c_int32,
                                 C.c_void_p, C.c_void_p]),
    "dqn_train_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_void_p, C.c_int32, C.c_void_p]),
    "dqn_get_train_q": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "dqn_train_step_sampled": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_uint64, C.c_int32, C.c_void_p]),
    "dqn_sync_target": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32]),
    "replay_create": (C.c_int, [C.c_int64, C.c_int32, C.c_int64, C.c_uint64, C.c_void_p, C.c_void_p,
                                C.POINTER(C.c_void_p)]),
    "replay_destroy": (C.c_int, [C.c_void_p]),
    "replay_push": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                              C.c_int32]),
    "replay_push_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "dqn_act_push_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_int32, C.c_float, C.c_uint64, C.c_int32, C.c_void_p,
                                    C.c_void_p]),
    "replay_flush": (C.c_int, [C.c_void_p, C.c_int32]),
    "replay_num_valid": (C.c_int64, [C.c_void_p]),
    "replay_sample_gather": (C.c_int, [C.c_void_p, C.c_int32, C.c_uint64, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "synth_frames": (C.c_int, [C.c_void_p, C.c_int64, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32,
                               C.c_uint32, C.c_uint32, C.c_void_p]),
    "synth_transitions": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_uint64,
                                    C.c_uint64, C.c_uint64, C.c_int32, C.c_uint32, C.c_uint32,
                                    C.c_uint32, C.c_void_p]),
    "dqn_envs_create": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_void_p)]),
    "dqn_envs_destroy": (C.c_int, [C.c_void_p]),
    "dqn_envs_arrays": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                  C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]),
    "dqn_envs_reset": (C.c_int, [C.c_void_p]),
    "dqn_envs_act": (C.c_int, [C.c_void_p, C.c_float, C.c_uint64, C.c_int32, C.c_int32]),
    "dqn_envs_observe": (C.c_int, [C.c_void_p]),
    "dqn_alg1_create": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(dqn_alg1_config), C.POINTER(C.c_void_p)]),
    "dqn_alg1_destroy": (C.c_int, [C.c_void_p]),
    "dqn_alg1_prepopulate": (C.c_int, [C.c_void_p, C.c_int64]),
    "dqn_alg1_run": (C.c_int, [C.c_void_p, C.c_int64]),
    "dqn_alg1_flush": (C.c_int, [C.c_void_p]),
    "dqn_alg1_stats": (C.c_int, [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                 C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    "dqn_profile_kernel_count": (C.c_int, []),
    "dqn_profile_kernel_name": (C.c_char_p, [C.c_int]),
    "dqn_profile_select": (C.c_int, [C.c_void_p, C.c_int]),
    "dqn_profile_select_every": (C.c_int, [C.c_void_p, C.c_int, C.c_int32]),
    "dqn_profile_read": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    "dqn_last_error": (C.c_char_p, []),
}

if not os.path.exists(LIB_PATH):
    raise ImportError("%s is missing: build it with `python -m paper_2111_01264_amd.build` "
                      "(there is no CPU fallback)" % LIB_PATH)
_lib = C.CDLL(LIB_PATH)
for _name, (_res, _args) in EXPORTS.items():
    _fn = getattr(_lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


def _check(rc):
    if rc != DQN_OK:
        raise DqnError(rc, _lib.dqn_last_error().decode())


def _ptr(t):
    """torch tensor (device) -> address, None -> NULL."""
    if t is None:
        return None
    assert t.is_contiguous(), "tensors handed to the library must be contiguous"
    return t.data_ptr()


def _stream(s):
    return None if s is None else s.cuda_stream


def _host(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data


def dqn_last_error():
    return _lib.dqn_last_error().decode()


def dqn_create(cfg: dqn_config, act_stream, train_stream):
    out = C.c_void_p()
    _check(_lib.dqn_create(C.byref(cfg), _stream(act_stream), _stream(train_stream), C.byref(out)))
    return out


def dqn_destroy(ctx):
    _check(_lib.dqn_destroy(ctx))


def dqn_num_params(ctx):
    return int(_lib.dqn_num_params(ctx))


def dqn_set_params(ctx, which, host_src):
    a, p = _host(host_src, np.float32)
    _check(_lib.dqn_set_params(ctx, which, p, a.size))


def dqn_get_params(ctx, which):
    out = np.empty(dqn_num_params(ctx), dtype=np.float32)
    _check(_lib.dqn_get_params(ctx, which, out.ctypes.data, out.size))
    return out


def dqn_act(ctx, states, W, epsilon, act_step, use_target, actions, q_out=None):
    _check(_lib.dqn_act(ctx, _ptr(states), W, epsilon, act_step, use_target, _ptr(actions), _ptr(q_out)))


def dqn_act_static(ctx, states, W, epsilon, act_step, use_target, actions, q_out=None):
    _check(_lib.dqn_act_static(ctx, _ptr(states), W, epsilon, act_step, use_target, _ptr(actions), _ptr(q_out)))


def dqn_train_step(ctx, s, a, r, s2, done, B, loss_out=None):
    _check(_lib.dqn_train_step(ctx, _ptr(s), _ptr(a), _ptr(r), _ptr(s2), _ptr(done), B, _ptr(loss_out)))


def dqn_train_step_sampled(ctx, rb, B, sample_step, prefetch_next, loss_out=None):
    _check(_lib.dqn_train_step_sampled(ctx, rb, B, sample_step, 1 if prefetch_next else 0, _ptr(loss_out)))


def dqn_get_train_q(ctx, B, A, double_dqn=False):
    q_on = np.empty((B, A), dtype=np.float32)
    q_nt = np.empty((B, A), dtype=np.float32)
    q_no = np.empty((B, A), dtype=np.float32) if double_dqn else None
    _check(_lib.dqn_get_train_q(ctx, q_on.ctypes.data, q_nt.ctypes.data,
                                q_no.ctypes.data if double_dqn else None))
    return q_on, q_nt, q_no


def dqn_sync_target(ctx, rb, blocking):
    _check(_lib.dqn_sync_target(ctx, rb, blocking))


def replay_create(capacity_frames, lanes, staging_per_lane, seed, push_stream, sample_stream):
    out = C.c_void_p()
    _check(_lib.replay_create(capacity_frames, lanes, staging_per_lane, seed, _stream(push_stream),
                              _stream(sample_stream), C.byref(out)))
    return out


def replay_destroy(rb):
    _check(_lib.replay_destroy(rb))


def replay_push(rb, lane, frames, actions, rewards, terminals, n):
    _check(_lib.replay_push(rb, lane, _ptr(frames), _ptr(actions), _ptr(rewards), _ptr(terminals), n))


def replay_push_step(rb, frames, actions, rewards, terminals):
    _check(_lib.replay_push_step(rb, _ptr(frames), _ptr(actions), _ptr(rewards), _ptr(terminals)))


def dqn_act_push_step(ctx, rb, push_frames, push_actions, push_rewards, push_terminals, states, W, epsilon,
                      act_step, use_target, actions, q_out=None):
    _check(_lib.dqn_act_push_step(ctx, rb, _ptr(push_frames), _ptr(push_actions), _ptr(push_rewards),
                                  _ptr(push_terminals), _ptr(states), W, epsilon, act_step, use_target,
                                  _ptr(actions), _ptr(q_out)))


def replay_flush(rb, blocking):
    _check(_lib.replay_flush(rb, blocking))


def replay_num_valid(rb):
    return int(_lib.replay_num_valid(rb))


def replay_sample_gather(rb, B, sample_step, idx_in, s, s2, a, r, done, idx_out=None):
    _check(_lib.replay_sample_gather(rb, B, sample_step, _ptr(idx_in), _ptr(s), _ptr(s2), _ptr(a),
                                     _ptr(r), _ptr(done), _ptr(idx_out)))


def synth_frames(dst, n, id0, id_step, seed, stream_tag, pix_threshold, background, stream):
    _check(_lib.synth_frames(_ptr(dst), n, id0, id_step, seed, stream_tag, pix_threshold, background,
                             _stream(stream)))


def synth_transitions(actions, rewards, terminals, n, id0, id_step, seed, num_actions, t_neg, t_pos,
                      t_term, stream):
    _check(_lib.synth_transitions(_ptr(actions), _ptr(rewards), _ptr(terminals), n, id0, id_step, seed,
                                  num_actions, t_neg, t_pos, t_term, _stream(stream)))


def dqn_envs_create(ctx, rb, W):
    out = C.c_void_p()
    _check(_lib.dqn_envs_create(ctx, rb, W, C.byref(out)))
    return out


def dqn_envs_destroy(e):
    _check(_lib.dqn_envs_destroy(e))


def dqn_envs_arrays(e, W, A):
    """numpy views of the pinned shared arrays: observations [W,84,84] u8, actions [W] i32, rewards [W] f32,
    terminals [W] u8, q [W,A] f32 (valid until dqn_envs_destroy)."""
    p = [C.c_void_p() for _ in range(5)]
    _check(_lib.dqn_envs_arrays(e, *[C.byref(x) for x in p]))
    spec = [(C.c_uint8, (W, 84, 84)), (C.c_int32, (W,)), (C.c_float, (W,)), (C.c_uint8, (W,)), (C.c_float, (W, A))]
    return tuple(np.ctypeslib.as_array(C.cast(x, C.POINTER(t)), shape=shape) for x, (t, shape) in zip(p, spec))


def dqn_envs_reset(e):
    _check(_lib.dqn_envs_reset(e))


def dqn_envs_act(e, epsilon, act_step, use_target, want_q=0):
    _check(_lib.dqn_envs_act(e, epsilon, act_step, use_target, want_q))


def dqn_envs_observe(e):
    _check(_lib.dqn_envs_observe(e))


def dqn_alg1_create(ctx, rb, cfg: dqn_alg1_config):
    out = C.c_void_p()
    _check(_lib.dqn_alg1_create(ctx, rb, C.byref(cfg), C.byref(out)))
    return out


def dqn_alg1_destroy(h):
    _check(_lib.dqn_alg1_destroy(h))


def dqn_alg1_prepopulate(h, timesteps):
    _check(_lib.dqn_alg1_prepopulate(h, timesteps))


def dqn_alg1_run(h, timesteps):
    _check(_lib.dqn_alg1_run(h, timesteps))


def dqn_alg1_flush(h):
    _check(_lib.dqn_alg1_flush(h))


def dqn_alg1_stats(h):
    t, na, nt, ep = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
    rs = C.c_double()
    _check(_lib.dqn_alg1_stats(h, C.byref(t), C.byref(na), C.byref(nt), C.byref(rs), C.byref(ep)))
    return {"t": t.value, "act_steps": na.value, "train_steps": nt.value, "reward_sum": rs.value, "episodes": ep.value}


def dqn_profile_kernel_count():
    return int(_lib.dqn_profile_kernel_count())


def dqn_profile_kernel_name(kernel_id):
    r = _lib.dqn_profile_kernel_name(kernel_id)
    return r.decode() if r else None


def dqn_profile_select(ctx, kernel_id):
    _check(_lib.dqn_profile_select(ctx, kernel_id))


def dqn_profile_select_every(ctx, kernel_id, every):
    _check(_lib.dqn_profile_select_every(ctx, kernel_id, every))


def dqn_profile_read(ctx):
    ms, n = C.c_double(), C.c_int64()
    _check(_lib.dqn_profile_read(ctx, C.byref(ms), C.byref(n)))
    return ms.value, n.value
