"""Pins for the oracle's replay memory: staging/flush (Section 3), sampling and the frame-stack
gather with terminal masking.  The gather is checked against an independent formulation: every
lane keeps its whole history in an unbounded list with an episode number per frame (cumulative
count of terminals), and a stacked frame survives iff its episode number equals the current one."""
import itertools

import numpy as np
import pytest

from oracle import philox
from oracle.replay import OracleReplay, FRAME


def frame_of(tag):
    f = np.zeros(FRAME, dtype=np.uint8)
    f[:] = tag % 251 + 1          # never zero, so a masked frame is distinguishable
    f[0] = tag % 256
    f[1] = (tag >> 8) % 256
    return f


class History:
    """Unbounded per-lane history with episode ids (independent formulation)."""

    def __init__(self, lanes, M):
        self.M = M
        self.h = [[] for _ in range(lanes)]     # (frame, a, r, d, episode)
        self.ep = [0] * lanes

    def append(self, lane, f, a, r, d):
        self.h[lane].append((f, a, r, d, self.ep[lane]))
        if d:
            self.ep[lane] += 1

    def visible(self, lane):
        return self.h[lane][-self.M:]

    def stack(self, lane, j):
        vis = self.visible(lane)
        cur_ep, next_ep = vis[j][4], vis[j + 1][4]
        s = np.stack([vis[j - 3 + k][0] if vis[j - 3 + k][4] == cur_ep else np.zeros(FRAME, np.uint8)
                      for k in range(4)])
        s2 = np.stack([vis[j - 2 + k][0] if vis[j - 2 + k][4] == next_ep else np.zeros(FRAME, np.uint8)
                       for k in range(4)])
        return s, s2, vis[j][1], vis[j][2], vis[j][3]


@pytest.mark.parametrize("lanes", [1, 2])
def test_gather_exhaustive_tiny_ring(lanes):
    N = 16
    M = N // lanes
    rng = np.random.default_rng(lanes)
    for trial in range(6):
        rep = OracleReplay(N, lanes, seed=1)
        hist = History(lanes, M)
        tag = 0
        # several flushes of ragged sizes, so heads wrap and lanes differ in fill
        for rnd in range(5):
            for lane in range(lanes):
                n = int(rng.integers(0, M))
                fs, acts, rews, terms = [], [], [], []
                for _ in range(n):
                    tag += 1
                    f, a, r, d = frame_of(tag), tag % 5, float(tag % 3 - 1), int(rng.uniform() < 0.3)
                    fs.append(f); acts.append(a); rews.append(r); terms.append(d)
                    hist.append(lane, f, a, r, d)
                if n:
                    rep.push(lane, np.stack(fs), acts, rews, terms)
            rep.flush()
            for lane in range(lanes):
                c = rep.count[lane]
                assert c == min(len(hist.h[lane]), M)
                for j in range(3, c - 1):
                    s, s2, a, r, done = rep.gather([lane * M + j])
                    ws, ws2, wa, wr, wd = hist.stack(lane, j)
                    assert np.array_equal(s.reshape(4, FRAME), ws)
                    assert np.array_equal(s2.reshape(4, FRAME), ws2)
                    assert (a[0], r[0], done[0]) == (wa, np.float32(wr), float(wd))


def test_every_terminal_placement_in_the_window():
    # 5-frame window t-3..t+1 at ages 3..7 of a 1-lane ring; all 2^5 terminal patterns on ages 3..7
    for pattern in itertools.product([0, 1], repeat=5):
        rep = OracleReplay(16, 1, seed=0)
        term = [0, 0, 0] + list(pattern) + [0]
        frames = np.stack([frame_of(i + 1) for i in range(9)])
        rep.push(0, frames, list(range(9)), [0.0] * 9, term)
        rep.flush()
        j = 6                                              # stack ages 3..6, next stack 4..7
        s, s2, a, r, done = rep.gather([j])
        s, s2 = s.reshape(4, FRAME), s2.reshape(4, FRAME)
        for k in range(4):
            keep = not any(term[v] for v in range(j - 3 + k, j))
            assert np.array_equal(s[k], frames[j - 3 + k] if keep else np.zeros(FRAME, np.uint8))
            keep2 = not any(term[v] for v in range(j - 2 + k, j + 1))
            assert np.array_equal(s2[k], frames[j - 2 + k] if keep2 else np.zeros(FRAME, np.uint8))
        assert np.array_equal(s[3], frames[6]) and np.array_equal(s2[3], frames[7])  # newest never masked
        assert done[0] == float(term[6]) and a[0] == 6


def test_pushes_invisible_until_flush():
    rep = OracleReplay(32, 2, seed=3)
    f = np.stack([frame_of(i) for i in range(10)])
    rep.push(0, f, [0] * 10, [0.0] * 10, [0] * 10)
    assert rep.num_valid() == 0 and rep.count == [0, 0]
    with pytest.raises(ValueError):
        rep.sample_indices(4, 0)
    rep.flush()
    assert rep.count == [10, 0] and rep.num_valid() == 6
    before = rep.sample_indices(8, 1).copy()
    s_before = rep.gather(before)[0].copy()
    rep.push(0, f, [1] * 10, [1.0] * 10, [1] * 10)        # staged while "training" runs
    rep.push(1, f, [1] * 10, [1.0] * 10, [1] * 10)
    assert np.array_equal(rep.sample_indices(8, 1), before)
    assert np.array_equal(rep.gather(before)[0], s_before)   # D unchanged during training
    rep.flush()
    assert rep.count == [16, 10] and rep.num_valid() == 12 + 6


def test_sampling_is_valid_uniform_and_a_pure_function():
    rep = OracleReplay(400, 4, seed=77)
    sizes = [100, 37, 4, 60]          # lane 2 holds no complete transition (needs >= 5 frames)
    for lane, n in enumerate(sizes):
        rep.push(lane, np.zeros((n, FRAME), np.uint8), [0] * n, [0.0] * n, [0] * n)
    rep.flush()
    V = rep.num_valid()
    assert V == 96 + 33 + 0 + 56
    idx = np.concatenate([rep.sample_indices(512, step) for step in range(40)])
    lane, j = idx // rep.M, idx % rep.M
    assert ((j >= 3) & (j <= np.array(rep.count)[lane] - 2)).all() and not (lane == 2).any()
    # brute-force re-derivation of one draw from the published generator outputs
    x0, x1, _, _ = philox.draw(77, philox.TAG_SAMPLE, 5, 9)
    k = (((x1 << 32) | x0) * V) >> 64
    flat = [(l, 3 + t) for l in range(4) for t in range(max(rep.count[l] - 4, 0))]
    assert rep.sample_indices(10, 5)[9] == flat[k][0] * rep.M + flat[k][1]
    # uniform over the V valid transitions
    pos = {lj: n for n, lj in enumerate(flat)}
    counts = np.bincount([pos[(int(a), int(b))] for a, b in zip(lane, j)], minlength=V)
    expect = idx.size / V
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert chi2 < V + 6 * np.sqrt(2 * V)
    assert np.array_equal(rep.sample_indices(64, 3), rep.sample_indices(64, 3))
    assert not np.array_equal(rep.sample_indices(64, 3), rep.sample_indices(64, 4))


def test_wraparound_overwrites_oldest():
    rep = OracleReplay(8, 1, seed=0)
    f = np.stack([frame_of(i + 1) for i in range(13)])
    rep.push(0, f[:6], list(range(6)), [0.0] * 6, [0] * 6)
    rep.flush()
    rep.push(0, f[6:], list(range(6, 13)), [0.0] * 7, [0] * 7)
    rep.flush()
    assert rep.count == [8] and rep.head == [13 % 8]
    # visible ages 0..7 are pushes 5..12
    s, s2, a, _, _ = rep.gather([3])
    assert a[0] == 8 and np.array_equal(s.reshape(4, FRAME), f[5:9])
    assert np.array_equal(s2.reshape(4, FRAME), f[6:10])
    with pytest.raises(ValueError):
        rep.gather([7])          # the newest frame has no successor yet
    with pytest.raises(ValueError):
        rep.gather([2])
