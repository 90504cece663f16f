"""Helpers shared by the GPU parity tests (marshalling only; no arithmetic of the method)."""
import numpy as np
import torch

import paper_2111_01264_amd as P
from datagen import synth


def make_cfg(A, max_batch=32, max_envs=8, precision=P.DQN_PRECISION_FP32, double_dqn=0, centered=1, seed=7):
    c = P.dqn_config()
    c.num_actions, c.max_batch, c.max_envs = A, max_batch, max_envs
    c.precision, c.double_dqn, c.centered = precision, double_dqn, centered
    c.gamma, c.huber_delta, c.lr, c.rms_alpha, c.rms_eps = 0.99, 1.0, 2.5e-4, 0.95, 0.01
    c.seed = seed
    return c


_KEEP = []


def dev(a):
    """Host array -> device tensor that stays alive until the next synchronisation: the library's
    streams are not torch's current stream, so a temporary must not go back to torch's caching
    allocator (and be overwritten by the next upload) while a kernel may still read it."""
    t = torch.as_tensor(np.ascontiguousarray(a)).cuda()
    if len(_KEEP) > 512:
        torch.cuda.synchronize()
        _KEEP.clear()
    _KEEP.append(t)
    return t


def rel_err(got, ref):
    """Norm-wise relative error: max|got - ref| / max(max|ref|, 1e-6)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-6))


def blob_slices(A):
    """name -> slice of the public parameter blob."""
    out, off = {}, 0
    for name, shape, _ in synth.layer_shapes(A):
        n = int(np.prod(shape))
        out[name + ".w"] = slice(off, off + n)
        out[name + ".b"] = slice(off + n, off + n + shape[0])
        off += n + shape[0]
    return out


def fill_replay_from_host(rb, seed, lanes, per_lane, A, chunk=500, p_neg=0.05, p_pos=0.05, p_term=0.001,
                          oracle=None):
    """Pushes `per_lane` generated experiences into every lane (frame id = t * lanes + lane),
    flushing after every chunk; mirrors the same pushes into `oracle` if given."""
    for lo in range(0, per_lane, chunk):
        n = min(chunk, per_lane - lo)
        for lane in range(lanes):
            ids = (np.arange(lo, lo + n, dtype=np.uint64) * np.uint64(lanes) + np.uint64(lane))
            f = synth.frames(seed, synth.STREAM_REPLAY, ids)
            a, r, d = synth.transitions(seed, ids, A, p_neg, p_pos, p_term)
            P.replay_push(rb, lane, dev(f), dev(a), dev(r), dev(d), n)
            if oracle is not None:
                oracle.push(lane, f, a, r, d)
        P.replay_flush(rb, 1)
        if oracle is not None:
            oracle.flush()
