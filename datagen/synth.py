"""Seeded synthetic inputs shaped like the paper's Atari workload (Section 5.1, Table 5).

This module only *generates inputs*: replay frames, rewards, terminals, stored actions, act-step
states and initial network parameters.  It contains none of the method's arithmetic (no network
math, no replay indexing, no action selection) and is the one module that both the CPU oracle's
tests and the HIP path's tests/bench may import.

Generator definition (all arithmetic modulo 2**64):

    mix64(z):  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9; z ^= z >> 27; z *= 0x94D049BB133111EB;
               z ^= z >> 31                         (the SplitMix64 output function)
    word(seed, stream, i, g) = mix64( mix64( mix64(seed + GAMMA*(stream+1)) + i ) + GAMMA*(g+1) )
    GAMMA = 0x9E3779B97F4A7C15

Frame `i`, pixel `p` (0..7055, row-major 84x84):  w = word(seed, stream, i, p // 2);
    w32 = (w >> 32*(p % 2)) & 0xFFFFFFFF;  pixel = (w32 & 0xFF) if (w32 >> 8) < PIX_T else 40
    with PIX_T = ceil(0.05 * 2**24): background byte 40, 5 % of pixels uniform in [0, 255].

Transition `i` metadata:  w = word(seed, STREAM_META, i, 0);
    reward bits  rb = w & 0xFFFFFF           -> -1 if rb < T_neg, +1 if rb >= 2**24 - T_pos, else 0
    terminal bits tb = (w >> 24) & 0xFFFFFF  -> 1 if tb < T_term
    action bits  ab = (w >> 48) & 0xFFFF     -> (ab * A) >> 16
    with T_x = floor(p_x * 2**24).

Synthetic environment (stands in for the Atari emulator, which is not available; Algorithm 1's "environment
instance ... for each sampler thread").  Environment j of W emits the observation sequence o_0, o_1, ..:
    o_n = frame(seed, STREAM_ENV, i) with i = n * W + j.
At its n-th step it receives an action a and answers with (r, d) from w = word(seed, STREAM_ENV_META, i, 0):
    good = (((w >> 48) & 0xFFFF) * A) >> 16;  r = reward bits of w as above if a == good, else 0;
    d = terminal bits of w as above (independent of a).
After d = 1 the next observation o_{n+1} opens a new episode.
"""
from __future__ import annotations

import math

import numpy as np

GAMMA = 0x9E3779B97F4A7C15
M1 = 0xBF58476D1CE4E5B9
M2 = 0x94D049BB133111EB
MASK64 = (1 << 64) - 1

FRAME_H = 84
FRAME_W = 84
FRAME_BYTES = FRAME_H * FRAME_W  # 7056
BACKGROUND = 40
PIX_T = math.ceil(0.05 * (1 << 24))  # 838861

STREAM_REPLAY = 0   # replay-ring frames
STREAM_META = 1     # reward / terminal / action of a stored transition
STREAM_ACT = 2      # states handed to the act step
STREAM_ENV = 3      # observations of the synthetic environments
STREAM_ENV_META = 4 # their rewards / terminals / rewarded actions


def _mix64(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    z ^= z >> np.uint64(30)
    z *= np.uint64(M1)
    z ^= z >> np.uint64(27)
    z *= np.uint64(M2)
    z ^= z >> np.uint64(31)
    return z


def _mix64_int(z: int) -> int:
    z &= MASK64
    z ^= z >> 30
    z = (z * M1) & MASK64
    z ^= z >> 27
    z = (z * M2) & MASK64
    z ^= z >> 31
    return z


def stream_key(seed: int, stream: int) -> int:
    """mix64(seed + GAMMA*(stream+1)) as a Python int."""
    return _mix64_int((seed + GAMMA * (stream + 1)) & MASK64)


def words(seed: int, stream: int, ids: np.ndarray, g: np.ndarray) -> np.ndarray:
    """word(seed, stream, i, g) for broadcastable uint64 arrays `ids` and `g`."""
    with np.errstate(over="ignore"):
        a = np.uint64(stream_key(seed, stream))
        b = _mix64(a + np.asarray(ids, dtype=np.uint64))
        return _mix64(b + np.uint64(GAMMA) * (np.asarray(g, dtype=np.uint64) + np.uint64(1)))


def frames(seed: int, stream: int, ids) -> np.ndarray:
    """[n, 84, 84] uint8 frames for the given frame ids."""
    ids = np.asarray(ids, dtype=np.uint64).reshape(-1)
    out = np.empty((ids.size, FRAME_BYTES), dtype=np.uint8)
    g = np.arange(FRAME_BYTES // 2, dtype=np.uint64)[None, :]
    chunk = 512
    for lo in range(0, ids.size, chunk):
        w = words(seed, stream, ids[lo:lo + chunk, None], g)             # [c, 3528]
        w32 = np.stack([w & np.uint64(0xFFFFFFFF), w >> np.uint64(32)], axis=-1)  # [c, 3528, 2]
        w32 = w32.reshape(w.shape[0], FRAME_BYTES)
        sel = (w32 >> np.uint64(8)) < np.uint64(PIX_T)
        val = (w32 & np.uint64(0xFF)).astype(np.uint8)
        out[lo:lo + chunk] = np.where(sel, val, np.uint8(BACKGROUND))
    return out.reshape(-1, FRAME_H, FRAME_W)


def thresholds(p_neg: float, p_pos: float, p_term: float):
    """Integer thresholds (T_neg, T_pos, T_term) on 24-bit draws."""
    s = 1 << 24
    return int(math.floor(p_neg * s)), int(math.floor(p_pos * s)), int(math.floor(p_term * s))


def transitions(seed: int, ids, num_actions: int, p_neg=0.05, p_pos=0.05, p_term=0.001):
    """(actions int32, rewards float32, terminals uint8) for the given transition ids."""
    ids = np.asarray(ids, dtype=np.uint64).reshape(-1)
    t_neg, t_pos, t_term = thresholds(p_neg, p_pos, p_term)
    w = words(seed, STREAM_META, ids, np.zeros(1, dtype=np.uint64))
    rb = (w & np.uint64(0xFFFFFF)).astype(np.int64)
    tb = ((w >> np.uint64(24)) & np.uint64(0xFFFFFF)).astype(np.int64)
    ab = ((w >> np.uint64(48)) & np.uint64(0xFFFF)).astype(np.int64)
    rewards = np.zeros(ids.size, dtype=np.float32)
    rewards[rb < t_neg] = -1.0
    rewards[rb >= (1 << 24) - t_pos] = 1.0
    terminals = (tb < t_term).astype(np.uint8)
    actions = ((ab * num_actions) >> 16).astype(np.int32)
    return actions, rewards, terminals


def env_frames(seed: int, num_envs: int, n: int) -> np.ndarray:
    """[W, 84, 84] uint8: observation o_n of every synthetic environment."""
    ids = np.uint64(n) * np.uint64(num_envs) + np.arange(num_envs, dtype=np.uint64)
    return frames(seed, STREAM_ENV, ids)


def env_outcomes(seed: int, num_envs: int, n: int, actions, num_actions: int, p_neg=0.05, p_pos=0.05, p_term=0.001):
    """(rewards float32 [W], terminals uint8 [W]) of every synthetic environment's n-th step under `actions`."""
    ids = np.uint64(n) * np.uint64(num_envs) + np.arange(num_envs, dtype=np.uint64)
    t_neg, t_pos, t_term = thresholds(p_neg, p_pos, p_term)
    w = words(seed, STREAM_ENV_META, ids, np.zeros(1, dtype=np.uint64))
    rb = (w & np.uint64(0xFFFFFF)).astype(np.int64)
    tb = ((w >> np.uint64(24)) & np.uint64(0xFFFFFF)).astype(np.int64)
    good = ((((w >> np.uint64(48)) & np.uint64(0xFFFF)).astype(np.int64)) * num_actions) >> 16
    r = np.zeros(num_envs, dtype=np.float32)
    r[rb < t_neg] = -1.0
    r[rb >= (1 << 24) - t_pos] = 1.0
    r[np.asarray(actions, dtype=np.int64) != good] = 0.0
    return r, (tb < t_term).astype(np.uint8)


def act_states(seed: int, step: int, num_envs: int) -> np.ndarray:
    """[W, 4, 84, 84] uint8 states for act step `step` (frame id = (step*W + j)*4 + k)."""
    ids = (np.arange(num_envs * 4, dtype=np.uint64) + np.uint64(step * num_envs * 4))
    return frames(seed, STREAM_ACT, ids).reshape(num_envs, 4, FRAME_H, FRAME_W)


# Layer table of the Q-network (input [B,4,84,84]): (name, weight shape, fan_in).
def layer_shapes(num_actions: int):
    return [
        ("conv1", (32, 4, 8, 8), 4 * 8 * 8),
        ("conv2", (64, 32, 4, 4), 32 * 4 * 4),
        ("conv3", (64, 64, 3, 3), 64 * 3 * 3),
        ("fc1", (512, 3136), 3136),
        ("fc2", (num_actions, 512), 512),
    ]


def num_params(num_actions: int) -> int:
    n = 0
    for _, shape, _ in layer_shapes(num_actions):
        n += int(np.prod(shape)) + shape[0]
    return n


def init_params(seed: int, num_actions: int) -> np.ndarray:
    """Flat float32 blob [conv1.w, conv1.b, ..., fc2.w, fc2.b] (OIHW / [out,in]), every tensor
    uniform in (-1/sqrt(fan_in), +1/sqrt(fan_in))."""
    rng = np.random.default_rng(seed)
    parts = []
    for _, shape, fan_in in layer_shapes(num_actions):
        bound = 1.0 / math.sqrt(fan_in)
        parts.append(rng.uniform(-bound, bound, size=int(np.prod(shape))).astype(np.float32))
        parts.append(rng.uniform(-bound, bound, size=shape[0]).astype(np.float32))
    return np.concatenate(parts)


# ---- inputs on which no ReLU can change state under operand rounding ---------------------------------------

def block_frames(seed: int, n: int) -> np.ndarray:
    """[n, 84, 84] uint8 frames with large-scale structure: a random 4x4 grid of 21x21-pixel blocks at brightness
    0 / 48 / 96 / 144, plus per-pixel noise uniform in [0, 63] (numpy default_rng(seed)).  Windows of every conv
    layer then see clearly different sums at different positions (relative spread over the pixels of a channel of
    roughly 15 % / 10 % / 6 % after conv1 / conv2 / conv3 with margin_params below)."""
    rng = np.random.default_rng(seed)
    base = rng.integers(0, 4, size=(n, 4, 4), dtype=np.int64) * 48
    noise = rng.integers(0, 64, size=(n, FRAME_H, FRAME_W), dtype=np.int64)
    return (np.repeat(np.repeat(base, 21, axis=1), 21, axis=2) + noise).astype(np.uint8)


MARGIN_BIAS = 0.5
MARGIN_SCALE = {"conv1": 0.25, "conv2": 0.2, "conv3": 0.1, "fc1": 0.02, "fc2": 0.02}


def margin_params(seed: int, num_actions: int, split_channels: bool) -> np.ndarray:
    """Parameter blob for which every hidden pre-activation is at least MARGIN_BIAS away from zero on ANY
    non-negative input, by construction: hidden channel o has sign s_o (+1; with split_channels -1 for odd o), bias
    s_o * MARGIN_BIAS and weights s_o * |w| * scale with w from init_params(seed) -- a channel's weighted sum of
    non-negative inputs has the sign of its bias.  Odd channels are then switched off for every input, even ones
    are on.  fc2 keeps mixed signs (scaled so that |Q| stays well below the reward magnitudes used with it)."""
    theta = init_params(seed, num_actions).copy()
    off = 0
    for name, shape, _ in layer_shapes(num_actions):
        n = int(np.prod(shape))
        w = theta[off:off + n].reshape(shape[0], -1)
        if name == "fc2":
            w *= np.float32(MARGIN_SCALE[name])
        else:
            sign = np.ones(shape[0], dtype=np.float32)
            if split_channels:
                sign[1::2] = -1.0
            w[:] = np.abs(w) * np.float32(MARGIN_SCALE[name]) * sign[:, None]
            theta[off + n:off + n + shape[0]] = sign * np.float32(MARGIN_BIAS)
        off += n + shape[0]
    return theta
