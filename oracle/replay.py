"""CPU oracle of the replay memory D: lanes, staging, flush, sampling, frame-stack gather.
TEST INFRASTRUCTURE ONLY.

Follows Section 2.1 (experiences (s_t, a_t, r_t, s_{t+1}) buffered in D and "sampled randomly")
and Section 3 (experiences collected while training runs are held in temporary buffers and moved
into D only at the synchronisation point, so D is constant during training; Algorithm 1's
"flush all sampler threads' temporary buffers" step).  The paper does not say how a state is
assembled from stored frames; the reading taken here:

  * D holds single 84x84 uint8 frames o_t with (a_t, r_t, d_t); d_t = 1 iff the episode ended
    after a_t.  D is split into L lanes (one per sampler); lane l owns M = N/L slots and is a ring
    with write head h_l and fill count c_l = min(flushed, M).
  * The age index j in [0, c_l) counts from the oldest visible frame of the lane; it lives in
    slot (h_l - c_l + j) mod M.  A global index is l*M + j.
  * State s_t is the stack (o_{t-3}, o_{t-2}, o_{t-1}, o_t); a frame o_u of the stack is replaced
    by zeros if a terminal flag d_v = 1 lies in u <= v < t (it belongs to an earlier episode).
    s_{t+1} is the same rule one step later.  The most recent frame is never masked.
  * A transition at age j can be sampled iff 3 <= j <= c_l - 2.  With v_l = max(c_l - 4, 0) and
    V = sum_l v_l, draw k = floor(u64 * V / 2**64) from the counter-based generator (u64 = x1:x0)
    and walk the lanes in order: the lane with prefix_l <= k < prefix_l + v_l, j = 3 + k - prefix_l.
"""
from __future__ import annotations

import numpy as np

from . import philox

FRAME = 84 * 84


class OracleReplay:
    def __init__(self, capacity_frames: int, lanes: int, seed: int):
        assert capacity_frames % lanes == 0
        self.N, self.L, self.M = capacity_frames, lanes, capacity_frames // lanes
        self.seed = seed
        self.frames = np.zeros((self.N, FRAME), dtype=np.uint8)
        self.actions = np.zeros(self.N, dtype=np.int32)
        self.rewards = np.zeros(self.N, dtype=np.float32)
        self.terminals = np.zeros(self.N, dtype=np.uint8)
        self.head = [0] * lanes
        self.count = [0] * lanes
        self.staged = [[] for _ in range(lanes)]   # per lane: list of (frame, a, r, d)

    # -- Section 3: temporary buffers, invisible to sampling until the flush -----------------
    def push(self, lane, frames, actions, rewards, terminals):
        frames = np.asarray(frames, dtype=np.uint8).reshape(-1, FRAME)
        for i in range(frames.shape[0]):
            self.staged[lane].append((frames[i].copy(), int(actions[i]), float(rewards[i]),
                                      int(terminals[i])))

    def flush(self):
        for lane in range(self.L):
            for f, a, r, d in self.staged[lane]:
                slot = lane * self.M + self.head[lane]
                self.frames[slot] = f
                self.actions[slot] = a
                self.rewards[slot] = r
                self.terminals[slot] = d
                self.head[lane] = (self.head[lane] + 1) % self.M
                self.count[lane] = min(self.count[lane] + 1, self.M)
            self.staged[lane] = []

    # -- indexing ------------------------------------------------------------------------------
    def slot_of(self, lane: int, j: int) -> int:
        return lane * self.M + (self.head[lane] - self.count[lane] + j) % self.M

    def num_valid(self) -> int:
        return sum(max(c - 4, 0) for c in self.count)

    def sample_indices(self, B: int, sample_step: int) -> np.ndarray:
        """Global indices l*M + j of B transitions drawn uniformly with replacement."""
        V = self.num_valid()
        if V <= 0:
            raise ValueError("replay memory holds no complete transition")
        out = np.empty(B, dtype=np.int64)
        for i in range(B):
            x0, x1, _, _ = philox.draw(self.seed, philox.TAG_SAMPLE, sample_step, i)
            k = (((x1 << 32) | x0) * V) >> 64
            for lane in range(self.L):
                v = max(self.count[lane] - 4, 0)
                if k < v:
                    out[i] = lane * self.M + 3 + k
                    break
                k -= v
        return out

    # -- frame-stack gather with terminal masking -------------------------------------------
    def gather(self, idx):
        idx = np.asarray(idx, dtype=np.int64)
        B = idx.size
        s = np.zeros((B, 4, FRAME), dtype=np.uint8)
        s2 = np.zeros((B, 4, FRAME), dtype=np.uint8)
        a = np.zeros(B, dtype=np.int32)
        r = np.zeros(B, dtype=np.float32)
        done = np.zeros(B, dtype=np.float32)
        for b in range(B):
            lane, j = divmod(int(idx[b]), self.M)
            if not (0 <= lane < self.L and 3 <= j <= self.count[lane] - 2):
                raise ValueError("index %d is not a complete transition" % idx[b])
            term = lambda age: int(self.terminals[self.slot_of(lane, age)])
            for k in range(4):
                u = j - 3 + k                      # frame of s_t
                if not any(term(v) for v in range(u, j)):
                    s[b, k] = self.frames[self.slot_of(lane, u)]
                u2 = j - 2 + k                     # frame of s_{t+1}
                if not any(term(v) for v in range(u2, j + 1)):
                    s2[b, k] = self.frames[self.slot_of(lane, u2)]
            t = self.slot_of(lane, j)
            a[b] = self.actions[t]
            r[b] = self.rewards[t]
            done[b] = float(self.terminals[t])
        shape = (B, 4, 84, 84)
        return s.reshape(shape), s2.reshape(shape), a, r, done
